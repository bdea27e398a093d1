"""Mutation check of the oracle's pins (CPU only; run by hand: python tests/oracle_mutation_check.py [names]).

Plants one plausible mistake at a time (a dropped term, a wrong sign or index, a swapped operand, an
off-by-one in the step logic) in a COPY of oracle/adaeagle_oracle.c under a temporary directory, builds
the copy and runs the CPU pin tests against it.  Every mutant must be noticed by at least one pin; a
line ending in SURVIVED names a gap.  The file name keeps pytest from collecting it: the full run
rebuilds the oracle ~100 times and takes several minutes."""
import os
import shutil
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
WORK = None   # temporary directory of the run

# (name, old, new, occurrence index or None when unique)
M = [
    ("bf16_half_up", "u += 0x7fffu + lsb;", "u += 0x8000u;", None),
    ("bf16_half_down", "u += 0x7fffu + lsb;", "u += 0x7fffu;", None),
    ("argmax_last_tie", "if (x[i] > x[best]) best = i;", "if (x[i] >= x[best]) best = i;", None),
    ("round_half_up", "double r = nearbyint((double)y);", "double r = floor((double)y + 0.5);", None),
    ("clamp_no_upper", "if (r > (double)k_max) r = (double)k_max;", "", None),
    ("clamp_no_lower", "if (r < 0.0) r = 0.0;", "", None),
    ("silu_sign", "return x / (1.0f + expf(-x)); }", "return x / (1.0f + expf(x)); }", None),
    ("silu_sigmoid", "return x / (1.0f + expf(-x)); }", "return 1.0f / (1.0f + expf(-x)); }", None),
    ("bias_sign", "if (bias) v += bias[n];", "if (bias) v -= bias[n];", None),
    ("matmul_transposed", "wval(W, wdtype, base + (size_t)k);", "wval(W, wdtype, (size_t)k * (size_t)N + (size_t)n);", None),
    ("rms_no_mean", "const float ms = (float)(ss / (acc_t)d);", "const float ms = (float)(ss);", None),
    ("rms_no_eps", "const float r = 1.0f / sqrtf(ms + eps);", "const float r = 1.0f / sqrtf(ms);", None),
    ("rms_no_gain", "out[i] = (x[i] * r) * g[i];", "out[i] = (x[i] * r);", None),
    ("rms_no_sqrt", "const float r = 1.0f / sqrtf(ms + eps);", "const float r = 1.0f / (ms + eps);", None),
    ("rope_exponent", "-2.0 * (double)i / (double)head_dim", "-1.0 * (double)i / (double)head_dim", None),
    ("rope_sign1", "p[i] = a * c[i] - b * s[i];", "p[i] = a * c[i] + b * s[i];", None),
    ("rope_sign2", "p[i + half] = b * c[i] + a * s[i];", "p[i + half] = b * c[i] - a * s[i];", None),
    ("rope_pos_plus1", "const double ang = (double)pos * inv;", "const double ang = (double)(pos + 1) * inv;", None),
    ("rope_adjacent_pairs", "const float a = p[i], b = p[i + half];\n      p[i] = a * c[i] - b * s[i];\n      p[i + half] = b * c[i] + a * s[i];",
     "const float a = p[2 * i], b = p[2 * i + 1];\n      p[2 * i] = a * c[i] - b * s[i];\n      p[2 * i + 1] = b * c[i] + a * s[i];", None),
    ("attn_scale", "const float scale = 1.0f / sqrtf((float)head_dim);", "const float scale = 1.0f / (float)head_dim;", None),
    ("attn_gqa_map", "const int kh = h / group;", "const int kh = h % n_kv_heads;", None),
    ("attn_no_norm", "out[(size_t)h * head_dim + d] = (float)(a / den);", "out[(size_t)h * head_dim + d] = (float)(a);", None),
    ("attn_not_self", "m->V[li], pos0 + r + 1, H, Hk", "m->V[li], pos0 + r, H, Hk", None),
    ("attn_non_causal", "m->V[li], pos0 + r + 1, H, Hk", "m->V[li], pos0 + rows, H, Hk", None),
    ("resid1_dropped", "for (size_t i = 0; i < (size_t)rows * d; ++i) x[i] += o[i];", "for (size_t i = 0; i < (size_t)rows * d; ++i) x[i] = o[i];", 0),
    ("resid2_dropped", "for (size_t i = 0; i < (size_t)rows * d; ++i) x[i] += o[i];", "for (size_t i = 0; i < (size_t)rows * d; ++i) x[i] = o[i];", 1),
    ("swiglu_swapped", "g[i] = silu(g[i]) * u[i];", "g[i] = g[i] * silu(u[i]);", None),
    ("ffn_norm_wrong_gain", "lw->ffn_norm, d, c->rms_eps", "lw->attn_norm, d, c->rms_eps", None),
    ("k_not_rotated", "rope_apply(kk + (size_t)r * dkv, Hk, hd, cs, sn);", "", None),
    ("v_rotated", "rope_apply(kk + (size_t)r * dkv, Hk, hd, cs, sn);", "rope_apply(kk + (size_t)r * dkv, Hk, hd, cs, sn); rope_apply(vv + (size_t)r * dkv, Hk, hd, cs, sn);", None),
    ("k_cache_unrounded", "Kd[i] = c->wdtype == ORC_BF16 ? orc_bf16_round(kk[(size_t)r * dkv + i]) : kk[(size_t)r * dkv + i];", "Kd[i] = kk[(size_t)r * dkv + i];", None),
    ("no_final_norm", "orc_rmsnorm(x + (size_t)r * d, m->w.final_norm, d, c->rms_eps, feat + (size_t)r * d);", "memcpy(feat + (size_t)r * d, x + (size_t)r * d, sizeof(float) * d);", None),
    ("draft_cat_swapped", "memcpy(cat + (size_t)r * 2 * d, feats + (size_t)r * d, sizeof(float) * d);\n    embed(m, next_tok[r], cat + (size_t)r * 2 * d + d);",
     "memcpy(cat + (size_t)r * 2 * d + d, feats + (size_t)r * d, sizeof(float) * d);\n    embed(m, next_tok[r], cat + (size_t)r * 2 * d);", None),
    ("draft_prefill_cur_token", "draft_rows(m, m->F, ids + p0 + 1, drows, p0);", "draft_rows(m, m->F, ids + p0, drows, p0);", None),
    ("draft_catchup_cur_token", "m->hist + m->dlen + 1, catch_rows, m->dlen);", "m->hist + m->dlen, catch_rows, m->dlen);", None),
    ("draft_first_row_out", "memcpy(m->fhat, x + (size_t)(rows - 1) * d, sizeof(float) * d);", "memcpy(m->fhat, x, sizeof(float) * d);", None),
    ("draft_chain_slot", "draft_rows(m, feat, &m->draft_ids[i - 1], 1, n - 1 + i);", "draft_rows(m, feat, &m->draft_ids[i - 1], 1, n + i);", None),
    ("draft_catchup_first_feats", "draft_rows(m, m->F + (size_t)(m->nF - catch_rows) * d,", "draft_rows(m, m->F,", None),
    ("softmax_T_inverted", "p[i] = exp(((double)logits[i] - mx) / T);", "p[i] = exp(((double)logits[i] - mx) * T);", None),
    ("cdf_ge", "if (c > thr) return i;", "if (c >= thr) return i;", None),
    ("accept_le", "if (u[acc] < ratio) continue;", "if (u[acc] <= ratio) continue;", None),
    ("accept_ratio_inverted", "double ratio = ph[t] > 0.0 ? p[t] / ph[t] : 1.0;", "double ratio = p[t] > 0.0 ? ph[t] / p[t] : 1.0;", None),
    ("residual_sign", "ph[i] = p[i] - ph[i] > 0.0 ? p[i] - ph[i] : 0.0;", "ph[i] = ph[i] - p[i] > 0.0 ? ph[i] - p[i] : 0.0;", None),
    ("bonus_row_all_accepted", "softmax_T(target_logits + (size_t)k * vocab, vocab, temperature, p);", "softmax_T(target_logits + (size_t)(k > 0 ? k - 1 : 0) * vocab, vocab, temperature, p);", None),
    ("resample_uniform_index", "*bonus = orc_sample_inverse_cdf(tot > 0.0 ? ph : p, vocab, u[k]);", "*bonus = orc_sample_inverse_cdf(tot > 0.0 ? ph : p, vocab, u[acc]);", None),
    ("resample_from_target", "*bonus = orc_sample_inverse_cdf(tot > 0.0 ? ph : p, vocab, u[k]);", "*bonus = orc_sample_inverse_cdf(p, vocab, u[k]);", None),
    ("greedy_bonus_row", "*bonus = orc_argmax(target_logits + (size_t)acc * vocab, vocab);", "*bonus = orc_argmax(target_logits + (size_t)(acc > 0 ? acc - 1 : 0) * vocab, vocab);", None),
    ("greedy_stop_early", "while (acc < k && draft_ids[acc] ==", "while (acc < k - 1 && draft_ids[acc] ==", None),
    ("greedy_row_shift", "draft_ids[acc] == orc_argmax(target_logits + (size_t)acc * vocab, vocab)", "draft_ids[acc] == orc_argmax(target_logits + (size_t)(acc + 1) * vocab, vocab)", None),
    ("prefill_dlen", "m->dlen = n - 1;\n  m->hist[n]", "m->dlen = n;\n  m->hist[n]", None),
    ("ldlp_token_pending", "embed(m, m->hist[m->kv_len - 1], u);", "embed(m, m->hist[m->kv_len], u);", None),
    ("ldlp_order", "embed(m, m->hist[m->kv_len - 1], u);\n    memcpy(u + d, f, sizeof(float) * d);", "embed(m, m->hist[m->kv_len - 1], u + d);\n    memcpy(u, f, sizeof(float) * d);", None),
    ("ldlp_no_residual", "z[i] += silu(t[i]);", "z[i] = silu(t[i]);", None),
    ("ldlp_no_out_act", "a += (acc_t)silu(z[i]) * (acc_t)m->w.ldlp_w_out[i];", "a += (acc_t)z[i] * (acc_t)m->w.ldlp_w_out[i];", None),
    ("ldlp_first_feature", "const float *f = m->F + (size_t)(m->nF - 1) * d;", "const float *f = m->F;", None),
    ("ldlp_cls_last_tie", "if (cl == 0 || y > best_y)", "if (cl == 0 || y >= best_y)", None),
    ("ldlp_cls_no_bias", "const float y = (float)a + m->w.ldlp_b_out[cl];", "const float y = (float)a;", None),
    ("rollback_short", "m->kv_len = n + 1 + acc;", "m->kv_len = n + acc;", None),
    ("rollback_nF", "m->nF = acc + 1;", "m->nF = acc > 0 ? acc : 1;", None),
    ("ddd_strict", "m->cum_logp >= (double)c->ddd_threshold", "m->cum_logp > (double)c->ddd_threshold", None),
    ("ddd_one_more", "if (i >= k && !(c->ddd_enabled", "if (i > k && !(c->ddd_enabled", None),
    ("logp_sign", "m->cum_logp += ((double)lg[t] - mx) / T - log(se);", "m->cum_logp += ((double)lg[t] - mx) / T + log(se);", None),
    ("logp_no_T", "m->cum_logp += ((double)lg[t] - mx) / T - log(se);", "m->cum_logp += ((double)lg[t] - mx) - log(se);", None),
    ("logp_of_argmax", "m->cum_logp += ((double)lg[t] - mx) / T - log(se);", "m->cum_logp += 0.0 - log(se);", None),
    ("loss_asym_reversed", "tot += diff < 0.0 ? lambda * -diff : diff;", "tot += diff > 0.0 ? lambda * diff : -diff;", None),
    ("loss_no_mean", "return n > 0 ? tot / n : 0.0;", "return tot;", None),
    ("verify_block0", "m->block[0] = m->hist[m->kv_len];", "m->block[0] = m->hist[m->kv_len - 1];", None),
    ("step_tokens_shift", "for (int i = 0; i < acc; ++i) tokens_out[i] = m->block[1 + i];", "for (int i = 0; i < acc; ++i) tokens_out[i] = m->block[i];", None),
    ("override_ignored", "t = override_ids[i];\n    }", "}\n", None),
    ("draft_temp_ignored", "if (m->c.temperature <= 0.0f || !u_draft) return orc_argmax(lg, V);", "return orc_argmax(lg, V);", None),
    ("ar_no_advance", "m->kv_len += 1;\n    m->hist[m->kv_len] = orc_argmax", "m->hist[m->kv_len + 1] = orc_argmax", None),
]

M += [
    ("prefill_logits_first_row", "target_block(m, ids + p0, rows, p0, m->F, last ? rows - 1 : rows);", "target_block(m, ids + p0, rows, p0, m->F, last ? 0 : rows);", None),
    ("set_state_dlen", "m->dlen = kv_len - 1;\n  m->nF = 1;", "m->dlen = kv_len;\n  m->nF = 1;", None),
    ("kv_import_unrounded", "m->K[layer][i] = m->c.wdtype == ORC_BF16 ? orc_bf16_round(k[i]) : k[i];", "m->K[layer][i] = k[i];", None),
    ("draft_uniform_index", "orc_sample_inverse_cdf(p, V, u_draft[i]);", "orc_sample_inverse_cdf(p, V, u_draft[0]);", None),
    ("accept_uniform_index", "if (u[acc] < ratio) continue;", "if (u[0] < ratio) continue;", None),
    ("cdf_fallback_last", "  return last;\n}", "  return n - 1;\n}", None),
    ("rollback_hist_short", "for (int i = 0; i <= acc; ++i) m->hist[n + i] = m->block[i];", "for (int i = 0; i < acc; ++i) m->hist[n + i] = m->block[i];", None),
    ("ldlp_no_b_in", "matmul(m->w.ldlp_w_in, c->wdtype, h, in, u, 1, in, m->w.ldlp_b_in, z, h);", "matmul(m->w.ldlp_w_in, c->wdtype, h, in, u, 1, in, NULL, z, h);", None),
    ("ldlp_res_bias_shared", "m->w.ldlp_b_res + (size_t)r * h, t, h);", "m->w.ldlp_b_res, t, h);", None),
    ("ldlp_res_weight_shared", "(const void *)((const float *)m->w.ldlp_w_res + (size_t)r * h * h);", "(const void *)((const float *)m->w.ldlp_w_res);", None),
    ("ldlp_no_b_out", "const float y = (float)a + m->w.ldlp_b_out[0];", "const float y = (float)a;", None),
    ("draft_fc_no_bias", "matmul(m->w.draft_fc_w, c->wdtype, d, 2 * d, cat, rows, 2 * d, m->w.draft_fc_b, x, d);", "matmul(m->w.draft_fc_w, c->wdtype, d, 2 * d, cat, rows, 2 * d, NULL, x, d);", None),
    ("logp_not_reset", "  m->cum_logp = 0.0;\n  int i = 0;", "  int i = 0;", None),
    ("accept_draft_row0", "softmax_T(draft_logits + (size_t)acc * vocab, vocab, temperature, ph);", "softmax_T(draft_logits, vocab, temperature, ph);", None),
    ("accept_target_row0", "softmax_T(target_logits + (size_t)acc * vocab, vocab, temperature, p);", "softmax_T(target_logits, vocab, temperature, p);", None),
    ("attn_k_head0", "const float *kj = k + (size_t)j * kv_stride + (size_t)kh * head_dim;", "const float *kj = k + (size_t)j * kv_stride;", None),
    ("attn_v_head0", "(acc_t)v[(size_t)j * kv_stride + (size_t)kh * head_dim + d];", "(acc_t)v[(size_t)j * kv_stride + d];", None),
    ("draft_layer_is_last_target", "decoder_layer(m, &m->w.draft_layer, c->n_layers, x, rows, slot0);", "decoder_layer(m, &m->layers[c->n_layers - 1], c->n_layers, x, rows, slot0);", None),
    ("draft_rope_pos_plus1", "decoder_layer(m, &m->w.draft_layer, c->n_layers, x, rows, slot0);", "decoder_layer(m, &m->w.draft_layer, c->n_layers, x, rows, slot0 + 1);", None),
    ("draft_uses_draft_lm_norm", "matmul(m->w.lm_head, c->wdtype, V, d, m->fhat, 1, d, NULL, m->dlogits + (size_t)i * V, V);",
     "{ float *nf = (float *)malloc(sizeof(float) * d); orc_rmsnorm(m->fhat, m->w.final_norm, d, c->rms_eps, nf); matmul(m->w.lm_head, c->wdtype, V, d, nf, 1, d, NULL, m->dlogits + (size_t)i * V, V); free(nf); }", None),
    ("ar_uses_prev_token", "int32_t id = m->hist[m->kv_len];\n    target_block(m, &id, 1,", "int32_t id = m->hist[m->kv_len - 1];\n    target_block(m, &id, 1,", None),
    ("verify_pos_off", "target_block(m, m->block, n_rows, m->kv_len, m->F, 0);", "target_block(m, m->block, n_rows, m->kv_len + 1, m->F, 0);", None),
    ("chain_uses_true_feature", "memcpy(feat, m->fhat, sizeof(float) * d);", "memcpy(feat, m->F + (size_t)(m->nF - 1) * d, sizeof(float) * d);", None),
    ("chain_token_index", "draft_rows(m, feat, &m->draft_ids[i - 1], 1, n - 1 + i);", "draft_rows(m, feat, &m->draft_ids[0], 1, n - 1 + i);", None),
    ("cls_kmax_excluded", "for (int cl = 0; cl <= c->k_max; ++cl) {", "for (int cl = 0; cl < c->k_max; ++cl) {", None),
    ("wdtype_bf16_shift", "uint32_t u = (uint32_t)h << 16;\n  float f;", "uint32_t u = (uint32_t)h << 15;\n  float f;", None),
]

TESTS = ["tests/test_oracle_pieces.py", "tests/test_oracle_forward.py", "tests/test_oracle_accept.py",
         "tests/test_oracle_spec.py", "tests/test_host_logic.py"]


def run_one(i):
    name, old, new, occ = M[i]
    d = os.path.join(WORK, name)
    shutil.rmtree(d, ignore_errors=True)
    os.makedirs(d)
    shutil.copytree(os.path.join(ROOT, "oracle"), os.path.join(d, "oracle"), ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    shutil.copytree(os.path.join(ROOT, "tests"), os.path.join(d, "tests"), ignore=shutil.ignore_patterns("__pycache__"))
    shutil.copytree(os.path.join(ROOT, "paper_2412_18910_amd"), os.path.join(d, "paper_2412_18910_amd"),
                    ignore=shutil.ignore_patterns("*.so", "_build", "csrc", "__pycache__"))
    shutil.copy(os.path.join(ROOT, "bench.py"), d)
    src = os.path.join(d, "oracle", "adaeagle_oracle.c")
    s = open(src).read()
    cnt = s.count(old)
    if (occ is None and cnt != 1) or (occ is not None and cnt <= occ):
        return name, "BAD-PATTERN(%d)" % cnt
    if occ is None:
        s = s.replace(old, new)
    else:
        parts = s.split(old)
        s = old.join(parts[:occ + 1]) + new + old.join(parts[occ + 1:])
    open(src, "w").write(s)
    r = subprocess.run(["make", "-C", os.path.join(d, "oracle"), "-s", "-B"], capture_output=True, text=True)
    if r.returncode:
        return name, "BUILD-FAIL " + r.stderr[-200:]
    env = dict(os.environ, OMP_NUM_THREADS="2", PYTHONDONTWRITEBYTECODE="1")
    try:
        r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + TESTS, cwd=d, env=env,
                           capture_output=True, text=True, timeout=900)
    except subprocess.TimeoutExpired:
        return name, "killed (timeout)"
    tail = [l for l in r.stdout.splitlines() if l.startswith("FAILED") or " passed" in l or " failed" in l or "rror" in l]
    shutil.rmtree(d, ignore_errors=True)
    if r.returncode == 0:
        return name, "SURVIVED"
    return name, "killed: " + (tail[0][:150] if tail else r.stdout[-150:])


if __name__ == "__main__":
    sel = range(len(M)) if len(sys.argv) < 2 else [i for i in range(len(M)) if M[i][0] in sys.argv[1:]]
    WORK = tempfile.mkdtemp(prefix="oracle_mutants_")
    survived = 0
    try:
        with ThreadPoolExecutor(max_workers=3) as ex:
            for name, res in ex.map(run_one, sel):
                print(f"{name:28s} {res}", flush=True)
                survived += not res.startswith("killed")
    finally:
        shutil.rmtree(WORK, ignore_errors=True)
    print(f"{len(list(sel))} mutants, {survived} not killed")
    sys.exit(1 if survived else 0)
