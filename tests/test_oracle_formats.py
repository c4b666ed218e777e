"""Pins for the oracle's number formats and layout constants (CPU only)."""
import os

import numpy as np
import torch

from oracle import ess_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _constants():
    out = {}
    for line in open(os.path.join(GOLD, "paper_constants.txt")):
        line = line.split("#")[0].strip()
        if "=" in line:
            k, v = line.split("=")
            out[k.strip()] = float(v)
    return out


def test_e4m3_table_matches_library_cast():
    # independent pin: torch's float8_e4m3fn decode of all 256 patterns
    ref = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    tab = O.e4m3fn_table()
    assert np.array_equal(np.isnan(ref), np.isnan(tab))
    ok = ~np.isnan(ref)
    assert np.array_equal(ref[ok], tab[ok])
    assert np.array_equal(np.signbit(ref[ok]), np.signbit(tab[ok]))
    assert tab[0x7E] == 448.0 and tab[0x38] == 1.0 and tab[0x01] == 2.0 ** -9


def test_small_integers_are_exact_in_e4m3():
    ints = torch.arange(-16, 17, dtype=torch.float32)
    by = ints.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(O.decode_e4m3(by), ints.numpy().astype(np.float64))


def test_bf16_decode_matches_library():
    g = torch.Generator().manual_seed(3)
    bits = torch.randint(0, 65536, (4096,), generator=g).to(torch.int32)
    bits = bits[((bits >> 7) & 0xFF) != 0xFF]            # drop inf/nan patterns
    ref = bits.to(torch.int16).view(torch.bfloat16).to(torch.float64).numpy()
    got = O.decode_bf16(bits.numpy().astype(np.uint16))
    assert np.array_equal(ref, got)


def test_row_layouts_match_paper_sizes():
    c = _constants()
    # 656-byte entry = 512 one-byte latents + 4 four-byte scales + 64 two-byte rope values
    assert 512 * 1 + 4 * 4 + 64 * 2 == c["latent_entry_bytes"]
    # our quantised row: bf16 scales (648 bytes) padded to the paper's entry size
    assert O.LATENT_DIM + 4 * 2 + O.ROPE_DIM * 2 == 648 <= c["latent_entry_bytes"]
    # 16.8 % indexer share <=> 128-byte key + 4-byte scale per token beside a 656-byte entry
    assert abs(132 / (132 + 656) - c["indexer_cache_share"]) < 1e-3
    assert O.ROW_DIM * 2 == 1152


def test_quoted_gains_follow_from_table2():
    c = _constants()
    assert abs(c["t2_32k_mtp2_b160"] / c["t2_32k_mtp2_b52"] - 1 - c["gain_32k"]) < 1e-3
    assert abs(c["t2_128k_mtp2_b54"] / c["t2_128k_mtp2_b13"] - 1 - c["gain_128k"]) < 5e-3


def test_fp8_row_decode_matches_library_casts():
    from paper_2512_10576_amd import synth
    rows = synth.latent_rows_fp8(5, 7)
    got = O.decode_rows(rows.numpy(), O.FMT_FP8)
    lat = rows[:, :512].contiguous().view(torch.float8_e4m3fn).to(torch.float64).reshape(7, 4, 128)
    sc = rows[:, 512:520].contiguous().view(torch.bfloat16).to(torch.float64)
    rope = rows[:, 520:648].contiguous().view(torch.bfloat16).to(torch.float64)
    ref = torch.cat([(lat * sc.unsqueeze(-1)).reshape(7, 512), rope], dim=1).numpy()
    assert np.array_equal(got, ref)
    assert rows.shape[1] == 656 and int(rows[:, 648:].abs().sum()) == 0
    # quantisation is sane: dequantised latents are close to N(0,1) draws
    assert 0.8 < got[:, :512].std() < 1.2


def test_bf16_row_decode_matches_library_casts():
    from paper_2512_10576_amd import synth
    rows = synth.latent_rows_bf16(9, 5)
    got = O.decode_rows(rows.numpy(), O.FMT_BF16)
    ref = rows.contiguous().view(torch.bfloat16).to(torch.float64).numpy()
    assert got.shape == (5, 576) and np.array_equal(got, ref)
