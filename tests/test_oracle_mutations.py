"""The pins must have teeth: plant one plausible mistake at a time in a COPY of the oracle's C
source (a dropped term, a wrong sign or index, a transposed operand), build it on the CPU, and
check that the pin suite then fails.  The mistakes are planted in the oracle only; nothing here
touches the GPU."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "pfg_oracle.c")

MUTANTS = [
    ("forward_transposed_weight", "s += prev[i] * W[(size_t)i * dout + j];",
     "s += prev[i] * W[(size_t)j * din + i];"),
    ("forward_bias_dropped", "double s = bias ? bias[j] : 0.0;", "double s = 0.0;"),
    ("backward_transposed_weight", "s += g[j] * W[(size_t)i * dout + j];",
     "s += g[j] * W[(size_t)j * din + i];"),
    ("backward_mask_dropped", "pfgo_act_deriv(net->act, t.z[l - 2][i]) * s : s;", "s : s;"),
    ("backward_mask_wrong_layer", "pfgo_act_deriv(net->act, t.z[l - 2][i]) * s",
     "pfgo_act_deriv(net->act, t.z[l - 1][i < dout ? i : 0]) * s"),
    ("outer_product_wrong_input", "const double *ain = (l == 1) ? x : t.a[l - 2];",
     "const double *ain = (l == 1) ? x : t.z[l - 2];"),
    ("outer_product_transposed", "dW[l - 1][(size_t)i * dout + j] = ain[i] * g[j];",
     "dW[l - 1][(size_t)i * dout + j] = ain[i] * g[(i + j) % dout];"),
    ("head_sign", "p[label] -= 1.0;", "p[label] += 1.0;"),
    ("head_onehot_dropped", "p[label] -= 1.0;", ""),
    ("softmax_no_normalise", "for (int j = 0; j < n; ++j) p[j] /= den;", ""),
    ("gelu_deriv_sign", "return Phi + z * pdf;", "return Phi - z * pdf;"),
    ("gelu_deriv_term_dropped", "return Phi + z * pdf;", "return Phi;"),
    ("tanh_deriv", "return 1.0 - t * t;", "return 1.0 - t;"),
    ("relu_deriv_at_zero", "case PFGO_ACT_RELU: return z > 0.0 ? 1.0 : 0.0;",
     "case PFGO_ACT_RELU: return z >= 0.0 ? 1.0 : 0.0;"),
    ("softmax_jacobian_sign", "row[j] = p[k] * ((j == k ? 1.0 : 0.0) - p[j]);",
     "row[j] = p[k] * ((j == k ? 1.0 : 0.0) + p[j]);"),
    ("softmax_jacobian_transposed_scale", "row[j] = p[k] * ((j == k ? 1.0 : 0.0) - p[j]);",
     "row[j] = p[j] * ((j == k ? 1.0 : 0.0) - p[j]);"),
    ("jacobian_row_stacking", "body_row_input(net, x, t, row, J + ((size_t)b * S + s) * d0);",
     "body_row_input(net, x, t, row, J + ((size_t)s * B + b) * d0);"),
    ("seed_stride_ignored", "row = seeds + (size_t)b * seed_batch_stride + (size_t)s * dL;",
     "row = seeds + (size_t)s * dL;"),
    ("per_example_slice_offset",
     "dWi[l - 1] = dW[l - 1] + (size_t)i * net->dims[l - 1] * net->dims[l];",
     "dWi[l - 1] = dW[l - 1] + (size_t)(B - 1 - i) * net->dims[l - 1] * net->dims[l];"),
    ("loss_not_log", "if (loss) *loss = -log(p[label]);", "if (loss) *loss = -p[label];"),
    ("norm_bias_always_counted", "if (net->b && net->b[l - 1])\n      for (int j = 0; j < net->dims[l]; ++j) sq +=",
     "for (int j = 0; j < net->dims[l]; ++j) sq +="),
    ("norm_bias_never_counted", "sq += db[l - 1][j] * db[l - 1][j];", ";"),
    ("norm_not_rooted", "if (norm) *norm = sqrt(total);", "if (norm) *norm = total;"),
    ("norm_abs_instead_of_square", "sq += dW[l - 1][e] * dW[l - 1][e];", "sq += fabs(dW[l - 1][e]);"),
    ("tanh_second_deriv_sign", "return -2.0 * t * (1.0 - t * t);", "return 2.0 * t * (1.0 - t * t);"),
    ("gelu_second_deriv_constant", "return pdf * (2.0 - z * z);", "return pdf * (1.0 - z * z);"),
    ("hessian_curvature_term_dropped",
     "dgp[i] = dh * pfgo_act_deriv(net->act, zi) + h * pfgo_act_deriv2(net->act, zi) * dz[l - 2][i];",
     "dgp[i] = dh * pfgo_act_deriv(net->act, zi);"),
    ("hessian_curvature_uses_masked_cotangent",
     "h * pfgo_act_deriv2(net->act, zi) * dz[l - 2][i];",
     "gp[i] * pfgo_act_deriv2(net->act, zi) * dz[l - 2][i];"),
    ("hessian_tangent_of_activation", "da[l - 1][c] = (l < L) ? pfgo_act_deriv(net->act, t.z[l - 1][c]) * s : s;",
     "da[l - 1][c] = s;"),
    ("hessian_tangent_mask_dropped_in_reverse", "dgp[i] = dh * pfgo_act_deriv(net->act, zi) +",
     "dgp[i] = dh +"),
    ("hessian_direction_ignored", "(i == j ? 1.0 : 0.0) : da[l - 2][i];",
     "(i == 0 ? 1.0 : 0.0) : da[l - 2][i];"),
    ("hessian_seed_stacking", "double *Hbs = H + ((size_t)b * S + s) * d0 * d0;",
     "double *Hbs = H + ((size_t)s * B + b) * d0 * d0;"),
]


LSTM_SRC = os.path.join(ROOT, "oracle", "lstm_oracle.c")

WHILE_GRADS = "void lstmo_body_while_grads("
WHILE_NORMS = "void lstmo_body_while_grad_norm("

LSTM_MUTANTS = [
    ("norm_cross_term", "for (size_t e = 0; e < nW; ++e) s[0] += dW[e] * dW[e];",
     "for (size_t e = 0; e < nW; ++e) s[0] += dW[e] * dW[(e + 1) % nW];"),
    ("norm_bias_block_dropped", "if (norm) *norm = sqrt(s[0] + s[1] + s[2] + s[3]);",
     "if (norm) *norm = sqrt(s[0] + s[2] + s[3]);"),
    ("norm_blocks_swapped", "for (size_t e = 0; e < nWo; ++e) s[2] += dWout[e] * dWout[e];",
     "for (size_t e = 0; e < nWo; ++e) s[3] += dWout[e] * dWout[e];"),
    ("norm_stacking", "sq ? sq + 4 * i : NULL, norm ? norm + i : NULL,",
     "sq ? sq + 4 * (B - 1 - i) : NULL, norm ? norm + i : NULL,"),
    ("gate_order_g_and_f", "g = tanh(z[H + k]), f = sigmoid(z[2 * H + k]),",
     "g = tanh(z[2 * H + k]), f = sigmoid(z[H + k]),"),
    ("forget_gate_dropped", "const double c = f * (cprev ? cprev[k] : 0.0) + i * g;",
     "const double c = (cprev ? cprev[k] : 0.0) + i * g;"),
    ("output_gate_on_cell", "tp.h[(size_t)t * H + k] = o * tanh(c);", "tp.h[(size_t)t * H + k] = o * c;"),
    ("recurrent_rows_offset", "s += hprev[r] * net->W[(size_t)(dx + r) * G + col];",
     "s += hprev[r] * net->W[(size_t)r * G + col];"),
    ("bias_dropped", "double s = net->b ? net->b[col] : 0.0;", "double s = 0.0;"),
    ("initial_state_not_zero", "const double *cprev = t > 0 ? tp.c + (size_t)(t - 1) * H : NULL;   /* c_0 = 0 */",
     "const double *cprev = tp.c + (size_t)(t > 0 ? t - 1 : 0) * H;"),
    ("bptt_cell_path_dropped", "const double dct = dc[k] + dh[k] * o * (1.0 - tc * tc);",
     "const double dct = dh[k] * o * (1.0 - tc * tc);"),
    ("bptt_tanh_deriv", "const double dct = dc[k] + dh[k] * o * (1.0 - tc * tc);",
     "const double dct = dc[k] + dh[k] * o * (1.0 - tc);"),
    ("bptt_output_gate", "dz[3 * H + k] = dh[k] * tc * o * (1.0 - o);", "dz[3 * H + k] = dh[k] * o * (1.0 - o);"),
    ("bptt_input_gate_swapped", "dz[k] = dct * g * i * (1.0 - i);", "dz[k] = dct * i * i * (1.0 - i);"),
    ("bptt_forget_uses_current_cell", "dz[2 * H + k] = dct * (cprev ? cprev[k] : 0.0) * f * (1.0 - f);",
     "dz[2 * H + k] = dct * tp.c[(size_t)t * H + k] * f * (1.0 - f);"),
    ("bptt_cell_carry", "dc[k] = dct * f;", "dc[k] = dct;"),
    ("weights_not_summed_over_steps", "dW[(size_t)r * G + col] += xt[r] * dz[col];",
     "dW[(size_t)r * G + col] = xt[r] * dz[col];"),
    ("bias_not_summed_over_steps", "db[col] += dz[col];", "db[col] = dz[col];"),
    ("recurrent_grad_uses_current_state", "dW[(size_t)(dx + r) * G + col] += hprev[r] * dz[col];",
     "dW[(size_t)(dx + r) * G + col] += tp.h[(size_t)t * H + r] * dz[col];"),
    ("hidden_cotangent_transposed", "s += dz[col] * net->W[(size_t)(dx + r) * G + col];",
     "s += dz[col] * net->W[(size_t)(dx + col % H) * G + (r + (col / H) * H)];"),
    ("input_cotangent_wrong_step", "gx[(size_t)t * dx + r] = s;", "gx[(size_t)(T - 1 - t) * dx + r] = s;"),
    ("readout_cotangent", "s += gy[j] * net->Wout[(size_t)k * dy + j];", "s += gy[j] * net->Wout[(size_t)j * H + k];"),
    ("head_sign", "p[label] -= 1.0;", "p[label] += 1.0;"),
    ("jacobian_row_stacking", "J + ((size_t)b * S + s) * nx);", "J + ((size_t)s * B + b) * nx);"),
    ("seed_stride_ignored", "row = seeds + (size_t)b * seed_batch_stride + (size_t)s * dy;",
     "row = seeds + (size_t)s * dy;"),
    ("varlen_runs_one_step_too_many", "while (t < len) {", "while (t <= len - 1 + (len > 1)) {"),
    ("varlen_state_not_carried", "c[k] = f * c[k] + i * g;", "c[k] = i * g;"),
    ("varlen_recurrent_term_dropped",
     "for (int r = 0; r < H; ++r) s += h[r] * net->W[(size_t)(dx + r) * G + col];", ""),
    ("while_halting_test_strict", "score <= 0.0)) break;", "score < 0.0)) break;"),
    ("while_first_trip_unconditional", "if (!(t < len && t < max_steps && score <= 0.0)) break;",
     "if (t > 0 && !(t < len && t < max_steps && score <= 0.0)) break;"),
    ("while_cap_off_by_one", "t < max_steps && score", "t <= max_steps && score"),
    ("while_length_off_by_one", "if (!(t < len && t < max_steps", "if (!(t <= len - (len > 0) && t < max_steps"),
    ("while_score_offset_dropped", "double score = halt_c;", "double score = 0.0;"),
    ("while_score_reads_the_cell_state", "score += h[k] * halt_w[k];", "score += c[k] * halt_w[k];"),
    ("while_steps_stacking", "steps_out ? steps_out + i : NULL);", "steps_out ? steps_out + (B - 1 - i) : NULL);"),
    ("while_state_stacking", "halt_w, halt_c, h_out ? h_out + (size_t)i * net->H : NULL,",
     "halt_w, halt_c, h_out ? h_out + (size_t)(B - 1 - i) * net->H : NULL,"),
    ("varlen_sequence_offset", "X + (size_t)offsets[i] * net->dx, offsets[i + 1] - offsets[i],",
     "X + (size_t)offsets[i] * net->dx + (i > 0 ? net->dx : 0), offsets[i + 1] - offsets[i],"),
    # gradients through the while loop: mistakes planted in that function only
    ("while_grads_gate_history_not_indexed_by_trip", "gi[(size_t)t * H + k] = i;", "gi[k] = i;", WHILE_GRADS),
    ("while_grads_state_history_not_indexed_by_trip", "cs[(size_t)t * H + k] = c[k];", "cs[k] = c[k];", WHILE_GRADS),
    ("while_grads_sweep_over_the_cap", "for (t = T - 1; t >= 0; --t) {", "for (t = (T > 0 ? cap : 0) - 1; t >= 0; --t) {",
     WHILE_GRADS),
    ("while_grads_sweep_skips_the_first_trip", "for (t = T - 1; t >= 0; --t) {", "for (t = T - 1; t >= 1; --t) {",
     WHILE_GRADS),
    ("while_grads_cell_carry", "dc[k] = dct * f;", "dc[k] = dct;", WHILE_GRADS),
    ("while_grads_recurrent_rows_use_current_state", "const double *hprev = t > 0 ? hs + (size_t)(t - 1) * H : NULL;",
     "const double *hprev = hs + (size_t)t * H;", WHILE_GRADS),
    ("while_grads_forget_gate_uses_current_cell", "dz[2 * H + k] = dct * (cprev ? cprev[k] : 0.0) * f * (1.0 - f);",
     "dz[2 * H + k] = dct * cs[(size_t)t * H + k] * f * (1.0 - f);", WHILE_GRADS),
    ("while_grads_readout_uses_first_state", "dWout[(size_t)k * dy + j] = h[k] * gy[j];",
     "dWout[(size_t)k * dy + j] = hs[k] * gy[j];", WHILE_GRADS),
    ("while_grads_head_sign", "gy[label] -= 1.0;", "gy[label] += 1.0;", WHILE_GRADS),
    ("while_grads_halting_test_strict", "score <= 0.0)) break;", "score < 0.0)) break;", WHILE_GRADS),
    ("while_grads_cap_ignored", "if (!(t < len && t < max_steps && score <= 0.0)) break;",
     "if (!(t < len && score <= 0.0)) break;", WHILE_GRADS),
    ("while_grads_bias_not_summed", "db[col] += dz[col];", "db[col] = dz[col];", WHILE_GRADS),
    ("while_grads_weights_not_summed", "dW[(size_t)r * G + col] += xt[r] * dz[col];",
     "dW[(size_t)r * G + col] = xt[r] * dz[col];", WHILE_GRADS),
    ("while_grads_seed_transposed", "s += gy[j] * net->Wout[(size_t)k * dy + j];",
     "s += gy[j] * net->Wout[(size_t)((k * dy + j) % H) * dy + (k * dy + j) / H % dy];", WHILE_GRADS),
    ("while_grads_hidden_cotangent_through_input_rows", "s += dz[col] * net->W[(size_t)(dx + r) * G + col];",
     "s += dz[col] * net->W[(size_t)(r % dx) * G + col];", WHILE_GRADS),
    ("while_grads_stacking", "labels[i], dW ? dW + (size_t)i * nW : NULL,",
     "labels[i], dW ? dW + (size_t)(B - 1 - i) * nW : NULL,", WHILE_GRADS),
    ("while_grads_sequence_offset", "lstmo_body_while_grads(net, X + (size_t)offsets[i] * net->dx,",
     "lstmo_body_while_grads(net, X + (size_t)offsets[i] * net->dx + (i > 0 ? net->dx : 0),", WHILE_GRADS),
    # norms of the gradients through the while loop: mistakes planted in that function and its pfor
    ("while_norms_cross_term", "for (size_t e = 0; e < nW; ++e) s[0] += dW[e] * dW[e];",
     "for (size_t e = 0; e < nW; ++e) s[0] += dW[e] * dW[(e + 1) % nW];", WHILE_NORMS),
    ("while_norms_bias_block_dropped", "if (norm) *norm = sqrt(s[0] + s[1] + s[2] + s[3]);",
     "if (norm) *norm = sqrt(s[0] + s[2] + s[3]);", WHILE_NORMS),
    ("while_norms_blocks_swapped", "for (size_t e = 0; e < nWo; ++e) s[2] += dWout[e] * dWout[e];",
     "for (size_t e = 0; e < nWo; ++e) s[3] += dWout[e] * dWout[e];", WHILE_NORMS),
    ("while_norms_not_a_root", "if (norm) *norm = sqrt(s[0] + s[1] + s[2] + s[3]);",
     "if (norm) *norm = s[0] + s[1] + s[2] + s[3];", WHILE_NORMS),
    ("while_norms_cap_ignored", "lstmo_body_while_grads(net, x, len, max_steps, halt_w, halt_c, label, dW,",
     "lstmo_body_while_grads(net, x, len, len, halt_w, halt_c, label, dW,", WHILE_NORMS),
    ("while_norms_condition_dropped", "lstmo_body_while_grads(net, x, len, max_steps, halt_w, halt_c, label, dW,",
     "lstmo_body_while_grads(net, x, len, max_steps, NULL, halt_c, label, dW,", WHILE_NORMS),
    ("while_norms_stacking", "labels[i], sq ? sq + 4 * i : NULL, norm ? norm + i : NULL,",
     "labels[i], sq ? sq + 4 * (B - 1 - i) : NULL, norm ? norm + i : NULL,", WHILE_NORMS),
    ("while_norms_sequence_offset", "lstmo_body_while_grad_norm(net, X + (size_t)offsets[i] * net->dx,",
     "lstmo_body_while_grad_norm(net, X + (size_t)offsets[i] * net->dx + (i > 0 ? net->dx : 0),", WHILE_NORMS),
]


CONV_SRC = os.path.join(ROOT, "oracle", "conv_oracle.c")

CONV_MUTANTS = [
    ("norm_cross_term", "for (size_t e = 0; e < cnt[i]; ++e) s += dWc[i][e] * dWc[i][e];",
     "for (size_t e = 0; e < cnt[i]; ++e) s += dWc[i][e] * dWc[i][(e + 1) % cnt[i]];"),
    ("norm_conv_bias_dropped", "for (size_t e = 0; e < cnt[nc + i]; ++e) s += dbc[i][e] * dbc[i][e];", ""),
    ("norm_absent_conv_bias_counted", "if (net->bc && net->bc[i])\n      for (size_t e = 0; e < cnt[nc + i]; ++e)",
     "for (size_t e = 0; e < cnt[nc + i]; ++e)"),
    ("norm_absent_dense_bias_counted", "if (net->b && net->b[l])\n      for (size_t e = 0; e < cnt[2 * nc + L + l]; ++e)",
     "for (size_t e = 0; e < cnt[2 * nc + L + l]; ++e)"),
    ("norm_dense_columns_first", "if (sq) sq[nc + l] = s;", "if (sq) sq[l] = s;"),
    ("norm_dense_weights_of_wrong_layer", "for (size_t e = 0; e < cnt[2 * nc + l]; ++e) s += dW[l][e] * dW[l][e];",
     "for (size_t e = 0; e < cnt[2 * nc]; ++e) s += dW[0][e] * dW[0][e];"),
    ("norm_not_a_root", "if (norm) *norm = sqrt(total);", "if (norm) *norm = total;"),
    ("norm_stacking", "sq ? sq + (size_t)cols * i : NULL,", "sq ? sq + (size_t)cols * (B - 1 - i) : NULL,"),
    ("conv_filter_flipped", "const int yy = y + ky - p, xs = xx + kx - p;\n              if (yy < 0 || yy >= hi || xs < 0 || xs >= wi) continue;      /* zero padding */",
     "const int yy = y - ky + p, xs = xx - kx + p;\n              if (yy < 0 || yy >= hi || xs < 0 || xs >= wi) continue;"),
    ("conv_padding_off_by_one", "const int k = net->kernel[i], p = (k - 1) / 2;\n    const double *W = net->Wc[i];\n    const double *bias",
     "const int k = net->kernel[i], p = (k - 1) / 2 - 1;\n    const double *W = net->Wc[i];\n    const double *bias"),
    ("conv_weight_index_transposed",
     "s += in[((size_t)yy * wi + xs) * ci + c] * W[(((size_t)ky * k + kx) * ci + c) * co + o];\n            }\n          t.z",
     "s += in[((size_t)yy * wi + xs) * ci + c] * W[(((size_t)kx * k + ky) * ci + c) * co + o];\n            }\n          t.z"),
    ("conv_bias_dropped", "double s = bias ? bias[o] : 0.0;", "double s = 0.0;"),
    ("pool_takes_minimum", "if (a > best) { best = a; where = (int32_t)at; }",
     "if (best < 0.0 || a < best) { best = a; where = (int32_t)at; }"),
    ("pool_before_relu", "const double a = t.z[i][at] > 0.0 ? t.z[i][at] : 0.0;", "const double a = t.z[i][at];"),
    ("pool_window_stride", "const size_t at = ((size_t)(2 * y + dy) * wi + (2 * xx + dx)) * co + o;",
     "const size_t at = ((size_t)(y + dy) * wi + (xx + dx)) * co + o;"),
    ("flatten_order", "out[((size_t)y * wo + xx) * co + o] = best;", "out[((size_t)o * ho + y) * wo + xx] = best;"),
    ("unpool_to_whole_window", "if (t.z[i][at] > 0.0) dz[at] = dout_buf[cell];          /* relu'(z) at the chosen entry */",
     "if (t.z[i][at] > 0.0) { dz[at] = dout_buf[cell]; if (at >= (int32_t)co && t.z[i][at - co] > 0.0) dz[at - co] = dout_buf[cell]; }"),
    ("conv_relu_mask_dropped", "if (t.z[i][at] > 0.0) dz[at] = dout_buf[cell];", "dz[at] = dout_buf[cell];"),
    ("filter_gradient_shift", "s += in[((size_t)yy * wi + xs) * ci + c] * dz[((size_t)y * wi + xx) * co + o];",
     "s += in[((size_t)y * wi + xx) * ci + c] * dz[((size_t)yy * wi + xs) * co + o];"),
    ("conv_bias_gradient_not_summed", "for (int xx = 0; xx < wi; ++xx) s += dz[((size_t)y * wi + xx) * co + o];",
     "for (int xx = 0; xx < wi; ++xx) s = dz[((size_t)y * wi + xx) * co + o];"),
    ("input_cotangent_not_accumulated", "din[((size_t)yy * wi + xs) * ci + c] += s;", "din[((size_t)yy * wi + xs) * ci + c] = s;"),
    ("input_cotangent_filter_flipped",
     "s += dz[((size_t)y * wi + xx) * co + o] * W[(((size_t)ky * k + kx) * ci + c) * co + o];",
     "s += dz[((size_t)y * wi + xx) * co + o] * W[(((size_t)(k - 1 - ky) * k + (k - 1 - kx)) * ci + c) * co + o];"),
    ("dense_input_cotangent_masked", "gprev[r] = (l > 1) ? (t.dz[l - 2][r] > 0.0 ? s : 0.0) : s;",
     "gprev[r] = (t.dz[l > 1 ? l - 2 : 0][r < net->dims[1] ? r : 0] > 0.0 ? s : 0.0);"),
    ("dense_uses_preactivation", "const double *ain = (l == 1) ? t.flat : t.da[l - 2];",
     "const double *ain = (l == 1) ? t.flat : t.dz[l - 2];"),
    ("head_sign", "g[label] -= 1.0;", "g[label] += 1.0;"),
    ("per_example_slice_offset", "if (dWc && dWc[j]) dWci[j] = dWc[j] + (size_t)i * nW;",
     "if (dWc && dWc[j]) dWci[j] = dWc[j] + (size_t)(B - 1 - i) * nW;"),
]


COND_SRC = os.path.join(ROOT, "oracle", "cond_oracle.c")

COND_MUTANTS = [
    ("condition_not_strict", "c = s > 0.0;", "c = s >= 0.0;"),
    ("condition_flipped", "c = s > 0.0;", "c = s < 0.0;"),
    ("condition_offset_dropped", "double s = net->c0;\n    for (int k = 0; k < dT; ++k) s += t[k] * net->w[k];\n    c =",
     "double s = 0.0;\n    for (int k = 0; k < dT; ++k) s += t[k] * net->w[k];\n    c ="),
    ("condition_reads_one_component", "for (int k = 0; k < dT; ++k) s += t[k] * net->w[k];\n    c =",
     "for (int k = 0; k < 1; ++k) s += t[k] * net->w[k];\n    c ="),
    ("branches_swapped", "if (c)\n    mlp_forward(net->then_net, t, 0, r);\n  else\n    mlp_forward(net->else_net, t, 0, r);",
     "if (c)\n    mlp_forward(net->else_net, t, 0, r);\n  else\n    mlp_forward(net->then_net, t, 0, r);"),
    ("else_branch_is_then", "else\n    mlp_forward(net->else_net, t, 0, r);", "else\n    mlp_forward(net->then_net, t, 0, r);"),
    ("invariant_flag_ignored", "if (invariant < 0) {", "if (1) {"),
    ("invariant_flag_inverted", "c = invariant != 0;", "c = invariant == 0;"),
    ("shared_part_without_last_activation", "mlp_forward(net->pre, x, 1, t);", "mlp_forward(net->pre, x, 0, t);"),
    ("branch_with_last_activation", "mlp_forward(which ? net->then_net : net->else_net, t, 0, r);",
     "mlp_forward(which ? net->then_net : net->else_net, t, 1, r);"),
    ("body_branch_with_last_activation", "if (c)\n    mlp_forward(net->then_net, t, 0, r);", "if (c)\n    mlp_forward(net->then_net, t, 1, r);"),
    ("bias_dropped", "double z = b ? b[j] : 0.0;", "double z = 0.0;"),
    ("weight_transposed", "z += cur[k] * W[(size_t)k * dout + j];", "z += cur[k] * W[(size_t)j * din + k];"),
    ("hidden_activation_dropped", "nxt[j] = (l < m->L || last_act) ? act_value(m->act, z) : z;",
     "nxt[j] = (l == m->L && last_act) ? act_value(m->act, z) : z;"),
    ("branch_reads_input_not_shared_part", "condo_pre(net, x, t);\n  mlp_forward(which ? net->then_net",
     "condo_pre(net, x, t); memcpy(t, x, sizeof(double) * (size_t)(dT < net->pre->dims[0] ? dT : net->pre->dims[0]));\n  mlp_forward(which ? net->then_net"),
    ("row_stacking", "const int c = condo_body(net, X + i * d0, invariant, R + i * dout);",
     "const int c = condo_body(net, X + i * d0, invariant, R + (n - 1 - i) * dout);"),
    ("condition_stacking", "if (cond) cond[i] = c;", "if (cond) cond[n - 1 - i] = c;"),
    ("score_offset_dropped", "double s = net->c0;\n  for (int k = 0; k < dT; ++k) s += t[k] * net->w[k];\n  free(t);",
     "double s = 0.0;\n  for (int k = 0; k < dT; ++k) s += t[k] * net->w[k];\n  free(t);"),
    ("grad_pre_mask_dropped", "g[j] = last_act ? gout[j] * act_deriv(m->act, z[m->L][j]) : gout[j];", "g[j] = gout[j];"),
    ("grad_hidden_mask_dropped", "gp[i] = (l > 1) ? s * act_deriv(m->act, z[l - 1][i]) : s;", "gp[i] = s;"),
    ("grad_weight_columns_reversed", "for (int j = 0; j < dout; ++j) s += g[j] * W[(size_t)i * dout + j];",
     "for (int j = 0; j < dout; ++j) s += g[j] * W[(size_t)i * dout + (dout - 1 - j)];"),
    ("grad_head_sign", "g[label] -= 1.0;", "g[label] += 1.0;"),
    ("grad_outer_uses_layer_output", "dW[l - 1][(size_t)i * dout + j] = a[l - 1][i] * g[j];",
     "dW[l - 1][(size_t)i * dout + j] = a[l - 1][i] * a[l][j];"),
    ("grad_bias_scaled", "for (int j = 0; j < dout; ++j) db[l - 1][j] = g[j];",
     "for (int j = 0; j < dout; ++j) db[l - 1][j] = g[j] * a[l - 1][0];"),
    ("grad_relu_deriv_at_zero", "case CONDO_ACT_RELU: return z > 0.0 ? 1.0 : 0.0;",
     "case CONDO_ACT_RELU: return z >= 0.0 ? 1.0 : 0.0;"),
    ("grad_row_stacking", "w[q][l - 1] = dWs[q][l - 1] + (size_t)i * m->dims[l - 1] * m->dims[l];",
     "w[q][l - 1] = dWs[q][l - 1] + (size_t)(n - 1 - i) * m->dims[l - 1] * m->dims[l];"),
    ("grad_loss_of_class_zero", "if (loss) *loss = -log(g[label]);", "if (loss) *loss = -log(g[0]);"),
    ("grad_untaken_branch_gets_the_taken_one", "zero_grads(other, dW_then, db_then);",
     "zero_grads(other, dW_then, db_then); if (other->dims[1] == taken->dims[1]) memcpy(db_then[0], db_else[0], sizeof(double) * (size_t)other->dims[1]);"),
    ("grad_tanh_deriv", "case CONDO_ACT_TANH: { const double t = tanh(z); return 1.0 - t * t; }",
     "case CONDO_ACT_TANH: { const double t = tanh(z); return 1.0 - t; }"),
    ("gelu_is_tanh_form", "return z * 0.5 * (1.0 + erf(z / sqrt(2.0)));",
     "return z * 0.5 * (1.0 + tanh(0.7978845608 * (z + 0.044715 * z * z * z)));"),
]


def run_mutants(oracle, tmp_path, source, mutants, env_var, pins_file):
    """Build every mutant and run the pin file against it, a few at a time; returns the names of
    the mutants that survived (passed every pin)."""
    src = open(source).read()

    def planted(m):
        # a fourth entry names the function the mistake belongs to: only the text from there on is changed
        # (the others stop short of that function, which repeats lines of the reverse sweep above it)
        name, old, new = m[:3]
        start = src.index(m[3]) if len(m) > 3 else 0
        end = src.index(WHILE_GRADS) if len(m) == 3 and WHILE_GRADS in src else len(src)
        if len(m) > 3 and m[3] == WHILE_GRADS and WHILE_NORMS in src:
            end = src.index(WHILE_NORMS)
        assert src.count(old, start, end) >= 1, f"pattern for {name} not found in {os.path.basename(source)}"
        return src[:start] + src[start:end].replace(old, new) + src[end:]

    for m in mutants:
        planted(m)

    def one(m):
        name = m[0]
        mutated = tmp_path / f"{name}.c"
        mutated.write_text(planted(m))
        lib = tmp_path / f"lib{name}.so"
        oracle.compile_source(str(mutated), str(lib))
        env = dict(os.environ, OMP_NUM_THREADS="2")
        env[env_var] = str(lib)
        r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", pins_file),
                            "-x", "-q", "-p", "no:cacheprovider"],
                           env=env, cwd=ROOT, capture_output=True, text=True, timeout=600)
        return name, r.returncode, r.stdout[-1500:]

    with ThreadPoolExecutor(max_workers=6) as pool:
        results = list(pool.map(one, mutants))
    return [(name, out) for name, rc, out in results if rc == 0]


def test_dense_pins_catch_every_planted_mistake(tmp_path, oracle):
    survivors = run_mutants(oracle, tmp_path, SRC, MUTANTS, "PFG_ORACLE_LIB", "test_oracle_pins.py")
    assert not survivors, "mutants that passed every pin: " + ", ".join(n for n, _ in survivors)


def test_lstm_pins_catch_every_planted_mistake(tmp_path, oracle):
    survivors = run_mutants(oracle, tmp_path, LSTM_SRC, LSTM_MUTANTS, "PFG_LSTM_ORACLE_LIB",
                            "test_oracle_lstm_pins.py")
    assert not survivors, "mutants that passed every pin: " + ", ".join(n for n, _ in survivors)


def test_conv_pins_catch_every_planted_mistake(tmp_path, oracle):
    survivors = run_mutants(oracle, tmp_path, CONV_SRC, CONV_MUTANTS, "PFG_CONV_ORACLE_LIB",
                            "test_oracle_conv_pins.py")
    assert not survivors, "mutants that passed every pin: " + ", ".join(n for n, _ in survivors)


def test_cond_pins_catch_every_planted_mistake(tmp_path, oracle):
    survivors = run_mutants(oracle, tmp_path, COND_SRC, COND_MUTANTS, "PFG_COND_ORACLE_LIB",
                            "test_oracle_cond_pins.py")
    assert not survivors, "mutants that passed every pin: " + ", ".join(n for n, _ in survivors)


def test_the_unmutated_oracles_pass_their_pins():
    # the check above would be empty if the pin files failed for another reason
    for pins in ("test_oracle_pins.py", "test_oracle_lstm_pins.py", "test_oracle_conv_pins.py",
                 "test_oracle_cond_pins.py"):
        r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", pins), "-x",
                            "-q", "-p", "no:cacheprovider"], cwd=ROOT, capture_output=True, text=True,
                           timeout=600)
        assert r.returncode == 0, r.stdout[-1500:]
