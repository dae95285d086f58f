"""Comparison of the HIP path's outputs with the CPU oracle's, element by element.

Bar: the W_sub gather, d2t ids and top-k ids bit-exact -- except that a
top-k position whose two candidate tokens have oracle logits within TIE_TOL of each other is
exempt -- and logits / log-probs within ABS_TOL absolute.  The only arithmetic difference
between the two sides is the order of the fp32 additions (sequential on the CPU; per lane,
then a tree, or MFMA blocks on the GPU) and exp/log rounding, so the observed differences are
orders of magnitude below ABS_TOL; TIGHT_TOL is asserted too so a real defect that happens to
stay under 2e-2 still fails.
"""
import numpy as np
import torch

ABS_TOL = 2e-2    # required bound on |logit| and |log-prob| differences
TIE_TOL = 2e-2    # ids whose oracle logits differ by at most this may swap
TIGHT_TOL = 2e-3  # engineering bound: fp32 reordering over H <= 4096 terms with |z| up to ~100


def to_dev_bf16(a_u16: np.ndarray, device="cuda:0") -> torch.Tensor:
    """numpy uint16 bf16 bit patterns -> torch.bfloat16 device tensor with the same bits."""
    t = torch.from_numpy(np.ascontiguousarray(a_u16).view(np.int16)).to(device)
    return t.view(torch.bfloat16)


def dev_bits(t: torch.Tensor) -> np.ndarray:
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def check_head(gpu_ids, gpu_logp, ora, d2t, Vd_total_vocab=None, gpu_logits=None, gpu_lse=None, rows=None):
    """gpu_ids/gpu_logp: numpy [R,k]; ora: oracle HeadResult for the same rows (with .z).
    Returns a dict of observed maxima; raises AssertionError on a violation."""
    R, k = gpu_ids.shape
    d2t = np.asarray(d2t)
    t2d = {int(t): j for j, t in enumerate(d2t)}
    stats = dict(max_dlogp=0.0, max_dlogit=0.0, max_dlse=0.0, id_mismatch=0, id_mismatch_tight=0)
    for r in range(R):
        z = ora.z[r]
        for p in range(k):
            gt, ot = int(gpu_ids[r, p]), int(ora.ids[r, p])
            assert gt in t2d, "row %d pos %d: id %d is not in the draft vocabulary" % (r, p, gt)
            gj = t2d[gt]
            if gt != ot:
                gap = abs(float(z[gj]) - float(z[ora.draft_idx[r, p]]))
                stats["id_mismatch"] += 1
                if gap > 1e-4:
                    stats["id_mismatch_tight"] += 1
                assert gap <= TIE_TOL, "row %d pos %d: id %d vs oracle %d, logit gap %g" % (r, p, gt, ot, gap)
            # log-prob of the token the GPU reports, against the oracle's value for that token
            want = float(z[gj]) - float(ora.lse[r])
            d = abs(float(gpu_logp[r, p]) - want)
            stats["max_dlogp"] = max(stats["max_dlogp"], d)
        # the reported tokens are distinct and best-first
        assert len(set(int(x) for x in gpu_ids[r])) == k
        assert np.all(np.diff(gpu_logp[r]) <= 0)
    if gpu_logits is not None:
        stats["max_dlogit"] = float(np.max(np.abs(gpu_logits.astype(np.float64) - ora.z.astype(np.float64))))
    if gpu_lse is not None:
        stats["max_dlse"] = float(np.max(np.abs(gpu_lse.astype(np.float64) - ora.lse.astype(np.float64))))
    for key in ("max_dlogp", "max_dlogit", "max_dlse"):
        assert stats[key] <= ABS_TOL, (key, stats)
        assert stats[key] <= TIGHT_TOL, (key, stats)
    return stats
