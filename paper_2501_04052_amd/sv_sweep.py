"""Special-value selection (Sec. 4.2 of arxiv 2501.04052): quantization error of a tensor for every
allowed special-value pair, measured with the HIP encoder and decoder.

The paper picks the allowed special values per model by measuring the weight quantization error of
adding one pair to NVFP4 (lowest at +-5 for every model), then of adding a second pair on top of +-5
for weights (+-8 for most models, +-7 / +-9 for two).  `sweep` does the same measurement on any
device tensor: it encodes with `razer_quantize`, decodes with `razer_dequant` and reports the squared
error normalised to the error without any special value pair that helps (the largest error seen, i.e.
what plain NVFP4 under the same scales gives).  All arithmetic of the format runs in the library;
torch only forms the error sum.

    python -m paper_2501_04052_amd.sv_sweep            # synthetic Llama-shaped weight, prints both sweeps
"""
import torch

from . import binding as razer

# multiples of 0.5 the decoder's offset register can form (6 +- 3.5) that are not FP4 values (Sec. 4.4)
ALLOWED = (2.5, 3.5, 4.5, 5.0, 5.5, 6.5, 7.0, 7.5, 8.0, 8.5, 9.0, 9.5)


def quantization_error(x, fmt, sv, block=16):
    """Sum of squared differences between x and its RaZeR reconstruction (fp64 on the device)."""
    t = razer.razer_quantize(x, fmt, sv, block=block)
    xh = razer.razer_dequant(t, torch.float32)
    return float(((x.to(torch.float32).double() - xh.double()) ** 2).sum().item())


def sweep(x, fmt=razer.WEIGHT, first=None, block=16):
    """Error for every allowed pair.  first=None: one pair added to plain FP4 (weights: both pairs set
    to the same value); first=v: a second pair on top of +-v (weight format only).
    Returns {special value: error / largest error of the sweep}."""
    errs = {}
    for v in ALLOWED:
        if first is None:
            sv = (v, v) if fmt == razer.WEIGHT else (v, 0.0)
        else:
            if fmt != razer.WEIGHT or v == first:
                continue
            sv = (first, v)
        errs[v] = quantization_error(x, fmt, sv, block)
    worst = max(errs.values())
    return {v: e / worst for v, e in errs.items()}


def best_pairs(x, block=16):
    """The paper's two-step choice for a weight tensor: best single pair, then best second pair."""
    one = sweep(x, razer.WEIGHT, None, block)
    v0 = min(one, key=one.get)
    two = sweep(x, razer.WEIGHT, v0, block)
    v1 = min(two, key=two.get)
    return (v0, v1), one, two


def main():
    from . import synth
    w = torch.from_numpy(synth.weight(4096, 4096, seed=1000, outlier_frac=0.001)).cuda()
    (v0, v1), one, two = best_pairs(w)
    print("one pair added to FP4 (error relative to the worst pair):")
    for v, e in one.items():
        print("  +-%-4g %.4f" % (v, e))
    print("second pair on top of +-%g:" % v0)
    for v, e in two.items():
        print("  +-%-4g %.4f" % (v, e))
    print("chosen special values: +-%g, +-%g" % (v0, v1))


if __name__ == "__main__":
    main()
