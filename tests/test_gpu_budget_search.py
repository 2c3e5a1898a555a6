"""The token-budget search of the library (paper Sec. 3.3; supplementary search algorithm) against the
oracle, on the GPU machine as well.

The search is host code and needs no GPU; these are the library-versus-oracle cases of
test_budget_search.py collected a second time under the `gpu` marker, so that the run on the GPU machine,
which loads the library it ships, covers them too.  The pins of the oracle itself stay CPU-only.
"""
import pytest

from test_budget_search import (  # noqa: F401  (collected from this module under the marker below)
    test_library_operators_match_the_oracle_bit_for_bit,
    test_library_search_matches_the_oracle_bit_for_bit,
    test_library_search_rejects_bad_arguments,
)

pytestmark = pytest.mark.gpu
