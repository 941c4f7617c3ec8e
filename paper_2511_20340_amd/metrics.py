"""Reporting helpers that follow the paper's own accounting (Methods, "From Arithmetic Intensity to
SD Evaluation"): chip arithmetic intensity AI_c, redundancy ratio rho, cost factor p, efficiency
kappa, and the kappa-to-TPS conversion ratio theta of the model-size study.  Host-side arithmetic
on a handful of scalars; nothing here is on the hot path."""

MI355X_HBM_BPS = 8.0e12          # published HBM3E bandwidth
MI355X_BF16_FLOPS = 2.5e15       # published dense bf16 MFMA peak
MI355X_FP32_FLOPS = 157.3e12     # published fp32 vector peak


def model_ai(bytes_per_param=2.0):
    """AI_m = 2 M / (bytes * M): FLOP per byte of a decoder reading every weight once per token."""
    return 2.0 / bytes_per_param


def chip_ai(peak_flops, bandwidth_bytes):
    """AI_c = peak FLOP/s / memory bandwidth (the A100 example gives 152.86)."""
    return peak_flops / bandwidth_bytes


def redundancy_ratio(peak_flops, bandwidth_bytes, bytes_per_param=2.0):
    """rho = AI_c / AI_m: ideal batch size / upper bound of the batching speed-up."""
    return chip_ai(peak_flops, bandwidth_bytes) / model_ai(bytes_per_param)


def max_draft_budget(rho, batch):
    """The constraint r2 = k <= rho / bs of the budgeted objective."""
    return rho / batch


def cost_factor(m_shared, m_per_position, l_d, m_model):
    """p = 1 + (m_s + l_d * m_p) / M."""
    return 1.0 + (m_shared + l_d * m_per_position) / m_model


def kappa(accepted_per_step, l_d, k):
    """kappa = a * l_d / k; without a draft tree l_d == k and kappa is the mean number of tokens
    emitted per target call (1 for plain decoding)."""
    return accepted_per_step * l_d / k if k else 1.0


def theta(kappa_value, speedup):
    """kappa-to-TPS conversion ratio of the model-size study."""
    return kappa_value / speedup


def draft_param_counts(d, hq, hkv, hd, ffn, k):
    """(shared, per-position) parameter counts of the draft block: the positional FFN holds
    k * d^2 position-specific weights (+ k*d biases); everything else is shared."""
    shared = 4 * d * d + (hq + 2 * hkv) * hd * d + hq * hd * d + 3 * d * ffn + 4 * d + 5 * d
    per_pos = d * d + d
    return shared, per_pos


def target_param_count(L, d, hq, hkv, hd, ffn, vocab):
    per_layer = (hq + 2 * hkv) * hd * d + hq * hd * d + 3 * d * ffn + 2 * d
    return L * per_layer + 2 * vocab * d + d
