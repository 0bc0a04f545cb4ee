"""Float64 numpy evaluation of the textbook Adam / AdamW update -- a sanity reference that pins
the fp32 C oracle; never compared against the HIP path at ulp level.  TEST INFRASTRUCTURE.

Formula: Kingma & Ba, Algorithm 1 (the optimizer the paper adopts, Sec. II "LLM Training Stages")
with bias-corrected moments m_hat = m'/(1-beta1^t), v_hat = v'/(1-beta2^t) and
    p' = p*(1 - lr*wd) - lr * m_hat / (sqrt(v_hat) + eps)             (decoupled decay, AdamW)
    p' = p             - lr * m_hat / (sqrt(v_hat) + eps),  g += wd*p  (L2 mode)
applied to g = g16 / loss_scale (mixed precision, Sec. V-A "Workloads"; tensors of Table II).
"""
import numpy as np


def half_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def adam_step_f64(p, m, v, g16_bits, *, lr, beta1, beta2, eps, weight_decay, step, loss_scale,
                  l2_mode=False):
    """Returns (p', m', v') as float64 arrays; inputs are left alone.  The hyper-parameters are
    first rounded to fp32 (as the C ABI receives them), then everything is float64."""
    f = lambda x: np.float64(np.float32(x))
    lr, beta1, beta2, eps, wd, S = map(f, (lr, beta1, beta2, eps, weight_decay, loss_scale))
    p = np.asarray(p, dtype=np.float64)
    m = np.asarray(m, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    g = half_bits_to_f64(g16_bits) / S
    if l2_mode:
        g = g + wd * p
    m_new = beta1 * m + (1.0 - beta1) * g
    v_new = beta2 * v + (1.0 - beta2) * g * g
    m_hat = m_new / (1.0 - beta1 ** step)
    v_hat = v_new / (1.0 - beta2 ** step)
    upd = lr * m_hat / (np.sqrt(v_hat) + eps)
    p_new = (p if l2_mode else p * (1.0 - lr * wd)) - upd
    return p_new, m_new, v_new


def sqnorm_f64(g16_bits, loss_scale) -> float:
    g = half_bits_to_f64(g16_bits) / np.float64(np.float32(loss_scale))
    return float(np.sum(g * g, dtype=np.float64))
