"""Which layers share attention in the paper's models (Sec. 5.1, table "The configurations of the
directly sharing attention (DS) and LiSA models"; layer numbers there start from 1).

A pattern is a tuple of layer kinds in layer order, ready for ``lisa.DecodeStack``:
"std" = standard attention, "lisa" = LiSA layer, "share" = direct sharing (DS).  The table is
configuration data of the method; nothing here computes anything.
"""
from __future__ import annotations

from typing import Dict, Iterable, Tuple

STD, LISA, SHARE = "std", "lisa", "share"


def _runs(*spans) -> Tuple[int, ...]:
    """1-based layer numbers from (first, last) spans and single numbers."""
    out = []
    for s in spans:
        if isinstance(s, tuple):
            out.extend(range(s[0], s[1] + 1))
        else:
            out.append(s)
    return tuple(out)


def _pattern(n_layers: int, lisa: Iterable[int] = (), share: Iterable[int] = ()) -> Tuple[str, ...]:
    kinds = [STD] * n_layers
    for n in lisa:
        kinds[n - 1] = LISA
    for n in share:
        assert kinds[n - 1] == STD
        kinds[n - 1] = SHARE
    return tuple(kinds)


# LLaMA3-8B and LLaMA2-7B (32 layers) use the same layer sets; LiSA (27) is listed for LLaMA3-8B only.
_S17 = _runs(5, 6, (17, 31))
_S21 = _runs(4, 5, 7, 8, 10, 11, 13, 14, 16, 17, 19, 20, (22, 30))
_S27 = _runs((4, 30))
# LLaMA2-13B (40 layers)
_S22 = _runs(7, 8, (19, 38))
_S26 = _runs((7, 10), (18, 39))

PATTERNS: Dict[str, Tuple[str, ...]] = {
    "all_standard_32": _pattern(32),
    "lisa_17_of_32": _pattern(32, lisa=_S17),
    "lisa_21_of_32": _pattern(32, lisa=_S21),
    "lisa_27_of_32": _pattern(32, lisa=_S27),
    "lisa_sl_7_10_of_32": _pattern(32, lisa=_runs(5, 6, (17, 21)), share=_runs((22, 31))),
    "ds_17_of_32": _pattern(32, share=_S17),
    "ds_21_of_32": _pattern(32, share=_S21),
    "ds_27_of_32": _pattern(32, share=_S27),
    "all_standard_40": _pattern(40),
    "lisa_22_of_40": _pattern(40, lisa=_S22),
    "lisa_26_of_40": _pattern(40, lisa=_S26),
    "lisa_sl_10_12_of_40": _pattern(40, lisa=_runs(7, 8, (19, 26)), share=_runs((27, 38))),
    "ds_22_of_40": _pattern(40, share=_S22),
    "ds_26_of_40": _pattern(40, share=_S26),
}


def sharing_layers(pattern) -> int:
    return sum(k != STD for k in pattern)
