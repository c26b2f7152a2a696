"""The floating-point bars of the GPU parity tests, one constant per quantity (bit-exact quantities --
order, cumulative priority, lengths, compacted bytes -- need none).

IMPORTANCE_RTOL  the bar named for the importance scores: 1e-3 relative, element by element.
DECODE_ATOL      attention outputs in bf16 storage against the fp64 oracle: 2e-2 absolute on values of order one
                 (one bf16 rounding of the output, 2^-9 relative, plus bf16-rounded probabilities in the prefill
                 kernel's second product).
LSE_RTOL/ATOL    log-sum-exp of a causal row in natural-log units.  The logits are fp32 sums of 64 or 128 exact
                 bf16 products: relative error <= 128 * 2^-24 = 7.6e-6 of sum |q_i k_i| * |scale|, which stays
                 below 40 for the test inputs, i.e. <= 3e-4 absolute on a logit and therefore on the lse; exp2 and
                 log2 of the hardware add about 1e-6 relative (the rtol term).
MERGE_RTOL_BF16  merged rows are means rounded to bf16 from fp32 sums where the oracle rounds from fp64 sums: the
                 two roundings can land on neighbouring bf16 values, one ulp = 2^-7 relative.
MERGE_RTOL_F32   the same for fp32 storage: 2e-6 (a few fp32 ulps of accumulated sum).
MERGE_ATOL       means whose magnitude is below the accumulation error of their sum (cancelling rows; a slot that
                 collects thousands of rows): <= count * 2^-24 * max|x| / count-independent bound of about 1e-4
                 for |x| <= 8.
"""
IMPORTANCE_RTOL = 1e-3
DECODE_ATOL = 2e-2
LSE_RTOL = 1e-4
LSE_ATOL = 3e-4
MERGE_RTOL_BF16 = 2.0 ** -7
MERGE_RTOL_F32 = 2e-6
MERGE_ATOL = 1e-4
