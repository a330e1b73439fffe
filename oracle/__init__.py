"""CPU oracle for the zip2zip dynamic-vocabulary path (arxiv 2506.01084).

TEST INFRASTRUCTURE ONLY.  These are plain, slow, obviously-correct CPU
implementations written from the paper: token-level LZW with a maximum merge
size (section 2.1, "LZW Algorithm"), the parameter-free averaging hyper-encoder
(section 2.2; hyper-encoder ablation table, "Averaging" row), and the joint
logits / softmax over the base and hyper vocabularies (section 2.3, steps 7-9),
temperature sampling from that softmax (step 9) with a counter-based generator,
and the learned hyper-encoder (section 2.2; attention and transformer rows of the
ablation table) in its standard pre-norm reading.

Nothing in the product path (the HIP library and its Python binding) may
import or call this package; only the tests, the smoke check and the
`cpu_baseline` leg of the benchmark do.  It shares no code with the HIP path.

Parity pins (tests/test_oracle_*.py): the reconstructed "to be or not to be"
example of Fig. 1, round trips, M=1 identity, textbook LZW at M=inf, the
closed form on a constant sequence, structural codebook invariants, brute
force over all tiny inputs, exact-rational rounding checks, pooling closed
forms, logit linearity and log-sum-exp bounds, the generator's published
known-answer vectors and a chi-square test of the draws, the library's
transformer encoder layer and multi-head attention for the learned hyper-encoder
(its gradient: the library's reverse-mode differentiation of the same modules and
finite differences of the forward pass).  The only unpinned item is the
literal content of Fig. 1's table, which is absent from the paper's text: the
fixture for it is a reconstruction from the captions.
"""
from .lzw import (LZWStream, lzw_encode, lzw_decode, pack_entries,  # noqa: F401
                  ST_OK, ST_BAD_TOKEN, ST_BAD_CODE, ST_OVERFLOW)
from .embed import hyper_embed, pool_coefficients  # noqa: F401
from .logits import extended_logits  # noqa: F401
from .sampling import (extended_sample, kept_prefix, philox4x32_10, sample_row,  # noqa: F401
                       sample_row_truncated)
from .loss import extended_nll, extended_nll_backward, hyper_embed_backward  # noqa: F401
from .encoder import hyper_encode, hyper_encode_backward  # noqa: F401
from .numfmt import bf16_bits_to_f64, f64_to_bf16_bits, to_f64, round_to_storage  # noqa: F401
