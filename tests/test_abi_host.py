"""CPU-only tests of the C-ABI library: exported symbols, the host packer and its error paths.
No compute entry point is called here."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2308_07641_amd as tsvd
import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if header.endswith(".h"):
            text = open(os.path.join(ROOT, "include", header)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(tsvd_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert {"tsvd_pack", "tsvd_forward", "tsvd_forward_ex", "tsvd_free", "tsvd_ternarize", "tsvd_fit_scales",
            "tsvd_transition"} <= set(names)
    lib = ctypes.CDLL(tsvd.lib_path())
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/*.h but not exported"


def test_tuning_switches_are_explicit_and_the_library_ignores_the_environment(monkeypatch):
    """The selection rules can only be overridden by tsvd_tuning_set in this process; unknown names are refused."""
    lib = tsvd.load_library()
    assert lib.tsvd_tuning_set(b"TSVD_NO_SUCH_SWITCH", 1) == 1
    with pytest.raises(ValueError):
        tsvd.tsvd_tuning_set("TSVD_STAGE_MASK", 4)          # the stage mask is an argument of the diagnostic forward only
    tsvd.tsvd_tuning_set("TSVD_FP6", 0)
    tsvd.tsvd_tuning_reset()
    src = "".join(open(os.path.join(ROOT, "paper_2308_07641_amd", "csrc", f)).read()
                  for f in os.listdir(os.path.join(ROOT, "paper_2308_07641_amd", "csrc")))
    assert "getenv" not in src


def test_strerror_covers_all_codes():
    texts = [tsvd.tsvd_strerror(s) for s in range(7)]
    assert texts[0] == "ok" and len(set(texts)) == 7


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (4, 4, 4), (3, 5, 7), (16, 256, 16), (17, 257, 33),
                                   (256, 256, 512), (300, 70, 513), (5, 1000, 2)])
def test_pack_unpack_round_trip_is_bit_exact(M, N, K):
    i = workloads.make_inputs(M, N, K, 1, 0.5, 0.02, "f32", seed=M * 1000 + N * 10 + K)
    blob = tsvd.tsvd_pack_host(i.U, i.S, i.V)
    assert blob.nbytes == tsvd.tsvd_packed_bytes(M, K, N)
    U, S, V = tsvd.tsvd_unpack_host(blob)
    assert U.dtype == np.int8 and np.array_equal(U, i.U)
    assert V.dtype == np.int8 and np.array_equal(V, i.V)
    assert np.array_equal(S.view(np.uint32), i.S.view(np.uint32))
    assert set(np.unique(U)) <= {-1, 0, 1} and set(np.unique(V)) <= {-1, 0, 1}
    # packing is a pure function of its inputs
    assert np.array_equal(blob, tsvd.tsvd_pack_host(i.U, i.S, i.V))


def _sections(blob):
    """Reads the blob header (layout documented in csrc/tsvd_layout.h)."""
    h = np.frombuffer(blob[:256].tobytes(), dtype=np.int64)
    names = ("magic", "ver_hdr", "M", "K", "N", "Mp", "Kp", "Np", "off_S", "off_U", "off_V",
             "off_nnzU", "off_nnzV", "total", "nnzU", "nnzV")
    return dict(zip(names, h[:16].tolist()))


def test_two_bit_codes_and_counts():
    """2 bits per element (section "Connection with BNN"): 00 = 0, 01 = +1, 11 = -1, 10 unused;
    the per-tile counts sum to the addition count of supplement Table S1."""
    i = workloads.make_inputs(40, 300, 70, 1, 0.6, 0.02, "f32", seed=5)
    blob = tsvd.tsvd_pack_host(i.U, i.S, i.V)
    s = _sections(blob)
    assert (s["Mp"], s["Kp"], s["Np"]) == (256, 256, 512)
    assert s["nnzU"] == np.count_nonzero(i.U) and s["nnzV"] == np.count_nonzero(i.V)
    for off, end, ref, noff in ((s["off_U"], s["off_V"], i.U, s["off_nnzU"]),
                                (s["off_V"], s["off_nnzU"], i.V, s["off_nnzV"])):
        words = np.frombuffer(blob[off:end].tobytes(), dtype=np.uint32)
        codes = (words[:, None] >> (2 * np.arange(16, dtype=np.uint32))[None, :]) & 3
        counts = np.bincount(codes.ravel(), minlength=4)
        assert counts[2] == 0                                   # 10 is never produced
        assert counts[1] == np.count_nonzero(ref == 1)
        assert counts[3] == np.count_nonzero(ref == -1)
        ntiles = words.size // 256
        nnz = np.frombuffer(blob[noff:noff + 2 * ntiles].tobytes(), dtype=np.uint16)
        per_tile = (codes != 0).reshape(ntiles, -1).sum(axis=1)
        assert np.array_equal(nnz, per_tile)
        assert nnz.sum() == np.count_nonzero(ref)
    # storage really is 2 bits per (padded) element
    assert s["off_V"] - s["off_U"] == s["Mp"] * s["Kp"] // 4
    assert s["off_nnzU"] - s["off_V"] == s["Kp"] * s["Np"] // 4


def _code_at(words, tiles_per_strip, r, c):
    """Element (r, c) of a packed matrix from the documented position rule: tile (r / 16, c / 256) of
    256 words; inside it lane 16 g + i (i = row in the tile), word 2 h + v / 2 of the lane and bit
    2 (2 n + v % 2), where h = step of 128 columns, kk = column in the step, g = bit 6 of kk + 2 x bit 4,
    operand element e = 16 x bit 5 + low four bits, v = e / 8, n = e % 8."""
    i, cc = r & 15, c & 255
    h, kk = cc >> 7, cc & 127
    g = ((kk >> 6) & 1) | (((kk >> 4) & 1) << 1)
    e = (((kk >> 5) & 1) << 4) | (kk & 15)
    v, n = e >> 3, e & 7
    word = (16 * g + i) * 4 + 2 * h + (v >> 1)
    return (int(words[((r >> 4) * tiles_per_strip + (c >> 8)) * 256 + word]) >> (2 * (2 * n + (v & 1)))) & 3


def _rank_position(k, K):
    """Where rank index k is stored: the last, partly filled block of 128 rank positions keeps its valid indices in the
    positions of the first 32-index sub-steps (offset bits [u p a b n] -> position bits [a u b p n])."""
    if K % 128 == 0 or k // 128 != K // 128:
        return k
    j = k % 128
    u, p_, a, b, n = (j >> 6) & 1, (j >> 5) & 1, (j >> 4) & 1, (j >> 3) & 1, j & 7
    return (k - j) + (a << 6 | u << 5 | b << 4 | p_ << 3 | n)


@pytest.mark.parametrize("K", [70, 128, 200, 345, 9])
def test_element_position_rule_of_the_tile_format(K):
    """Kernels that read single codes (the grouped convolution) use this rule; it must agree with the packer.  The
    rank index goes through the position rule of the format; S sits at the same positions, zeros elsewhere."""
    i = workloads.make_inputs(40, 300, K, 1, 0.6, 0.02, "f32", seed=5)
    blob = tsvd.tsvd_pack_host(i.U, i.S, i.V)
    s = _sections(blob)
    Uw = np.frombuffer(blob[s["off_U"]:s["off_V"]].tobytes(), dtype=np.uint32)
    Vw = np.frombuffer(blob[s["off_V"]:s["off_nnzU"]].tobytes(), dtype=np.uint32)
    Sw = np.frombuffer(blob[s["off_S"]:s["off_S"] + 4 * s["Kp"]].tobytes(), dtype=np.float32)
    value = {0: 0, 1: 1, 3: -1}
    pos = [_rank_position(k, K) for k in range(K)]
    assert len(set(pos)) == K and max(pos) < s["Kp"]
    # valid indices of the last block fill the first sub-steps: position bits 5 (u) and 3 (p) in that order
    r = K % 128
    if r:
        steps = sorted({((q % 128) >> 5 & 1) * 2 + ((q % 128) >> 3 & 1) for q in pos[K - r:]})
        assert steps == list(range(-(-r // 32)))
    assert all(value[_code_at(Uw, s["Kp"] // 256, r_, pos[c])] == i.U[r_, c] for r_ in range(40) for c in range(K))
    assert all(value[_code_at(Vw, s["Np"] // 256, pos[r_], c)] == i.V[r_, c] for r_ in range(K) for c in range(0, 300, 7))
    assert all(Sw[pos[k]] == i.S[k] for k in range(K))
    assert np.count_nonzero(Sw) == np.count_nonzero(i.S)


def test_single_element_sets_exactly_its_code():
    U = np.zeros((20, 300), dtype=np.int8)
    V = np.zeros((300, 10), dtype=np.int8)
    S = np.ones(300, dtype=np.float32)
    base = tsvd.tsvd_pack_host(U, S, V)
    s = _sections(base)
    for (r, c, val, bits) in ((0, 0, 1, 1), (19, 299, -1, 2), (7, 131, 1, 1), (16, 256, -1, 2), (3, 260, 1, 1)):
        U2 = U.copy()
        U2[r, c] = val
        b2 = tsvd.tsvd_pack_host(U2, S, V)
        diff = np.flatnonzero(base != b2)
        # one code byte, the tile's count, and the header's total change; nothing else
        in_tiles = diff[(diff >= s["off_U"]) & (diff < s["off_V"])]
        assert in_tiles.size == 1
        assert bin(int(base[in_tiles[0]] ^ b2[in_tiles[0]])).count("1") == bits
        U3, _, _ = tsvd.tsvd_unpack_host(b2)
        assert np.array_equal(U3, U2)


def test_pack_rejects_bad_input_and_leaves_output_untouched():
    i = workloads.make_inputs(8, 8, 8, 1, 0.5, 0.02, "f32", seed=1)
    lib = tsvd.load_library()
    n = tsvd.tsvd_packed_bytes(8, 8, 8)
    blob = np.full(n, 0xAB, dtype=np.uint8)
    U = i.U.copy()
    U[3, 3] = 2
    rc = lib.tsvd_pack_host(U.ctypes.data, i.S.ctypes.data, i.V.ctypes.data, 8, 8, 8, blob.ctypes.data, n)
    assert rc == 2 and np.all(blob == 0xAB)
    V = i.V.copy()
    V[0, 7] = -128
    rc = lib.tsvd_pack_host(i.U.ctypes.data, i.S.ctypes.data, V.ctypes.data, 8, 8, 8, blob.ctypes.data, n)
    assert rc == 2 and np.all(blob == 0xAB)
    # null pointers, bad sizes, short buffer
    assert lib.tsvd_pack_host(None, i.S.ctypes.data, i.V.ctypes.data, 8, 8, 8, blob.ctypes.data, n) == 1
    assert lib.tsvd_pack_host(i.U.ctypes.data, i.S.ctypes.data, i.V.ctypes.data, 0, 8, 8, blob.ctypes.data, n) == 1
    assert lib.tsvd_pack_host(i.U.ctypes.data, i.S.ctypes.data, i.V.ctypes.data, 8, 8, 8, blob.ctypes.data, n - 1) == 1
    assert np.all(blob == 0xAB)
    assert tsvd.tsvd_packed_bytes(0, 1, 1) == 0 and tsvd.tsvd_packed_bytes(1, -1, 1) == 0


def test_unpack_detects_corruption():
    i = workloads.make_inputs(8, 8, 8, 1, 0.0, 0.02, "f32", seed=2)    # no zeros: every code is 01 or 11
    blob = tsvd.tsvd_pack_host(i.U, i.S, i.V)
    s = _sections(blob)
    bad = blob.copy()
    bad[0] ^= 0xFF                                                     # magic
    with pytest.raises(tsvd.TsvdError):
        tsvd.tsvd_unpack_host(bad)
    with pytest.raises(tsvd.TsvdError):
        tsvd.tsvd_unpack_host(blob[:100])
    # turn a +1 (01) into the unused code 10
    tiles = blob[s["off_U"]:s["off_V"]]
    pos = int(np.flatnonzero((tiles & 3) == 1)[0]) + s["off_U"]
    bad = blob.copy()
    bad[pos] = (bad[pos] & ~np.uint8(3)) | np.uint8(2)
    with pytest.raises(tsvd.TsvdError) as e:
        tsvd.tsvd_unpack_host(bad)
    assert e.value.status == 2
    # a code in the zero padding
    bad = blob.copy()
    bad[s["off_V"] - 1] |= 1
    with pytest.raises(tsvd.TsvdError):
        tsvd.tsvd_unpack_host(bad)


def test_no_gpu_calls_fail_cleanly_without_a_device():
    """tsvd_pack needs a device: without one it must return a status, not crash."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    i = workloads.make_inputs(4, 4, 4, 1, 0.5, 0.02, "f32", seed=3)
    with pytest.raises(tsvd.TsvdError) as e:
        tsvd.tsvd_pack(i.U, i.S, i.V)
    assert e.value.status == 4


def test_new_entry_points_validate_arguments_before_touching_a_device():
    """Argument checks of the transition and convolution calls come first: null pointers, sizes out
    of range and misaligned workspaces are TSVD_EINVAL (1) with no device work (this test runs
    without a GPU)."""
    lib = tsvd.load_library()
    buf = (ctypes.c_double * 64)()
    p = ctypes.addressof(buf)
    assert lib.tsvd_ternarize(None, 4, 1, 4, 0.5, p, 4, p, None) == 1
    assert lib.tsvd_ternarize(p, 0, 1, 4, 0.5, p, 4, p, None) == 1
    assert lib.tsvd_ternarize(p, 9000, 1, 9000, 0.5, p, 9000, p, None) == 1          # n > 8192
    assert lib.tsvd_ternarize(p, 4, 1, 3, 0.5, p, 4, p, None) == 1                   # stride < n
    assert lib.tsvd_fit_scales_workspace(0) == 0 and lib.tsvd_fit_scales_workspace(4096) == 0
    assert lib.tsvd_fit_scales_workspace(100) >= 100 * 100 * 8 + 100 * 8
    assert lib.tsvd_fit_scales(p, 4, p, p, 4, 4, 4, p, None, 0, None, None) == 1     # no workspace
    assert lib.tsvd_fit_scales(p, 2, p, p, 4, 4, 4, p, p, 1 << 20, None, None) == 1  # ldu < K
    assert lib.tsvd_residual(p, p, 4, p, p, 4, 0, 4, p, None, None) == 1             # K = 0
    assert lib.tsvd_leading_singular_pair_workspace(0, 5) == 0
    assert lib.tsvd_leading_singular_pair(p, 4, 4, 10, p, p, p, None, None, 0, None) == 1
    rank = ctypes.c_int64(0)
    assert lib.tsvd_transition(p, 4, 4, 0.5, 0.1, 0, p, p, p, ctypes.byref(rank), None, None) == 1   # max_rank = 0
    assert lib.tsvd_transition(p, 4, 4, 0.5, -1.0, 4, p, p, p, ctypes.byref(rank), None, None) == 1  # tol < 0
    assert lib.tsvd_conv2d_workspace_bytes(None, p, 1, 4, 4) == 0
    assert lib.tsvd_conv2d_forward(None, p, p, 1, 4, 4, None, p, 0, p, 0, None) == 1
    assert lib.tsvd_workspace_bytes_ex(None, 4, 0, 0) == 0
    assert lib.tsvd_forward_ex(None, p, 0, 0, 1, 1, None, p, 0, 1, None, 0, None) == 1


# ---- the denser code of U: five ternary elements per byte
def _dense_decode(blob, M, K):
    """The documented rule written out independently: group of five strips, 4 KiB per (group, tile column) as
    [4 chunks][64 lanes][16 bytes]; byte j of a lane = sum_i trit(5 j + i) 3^i over the lane's codes q = 64 t + 16 w + n
    (strip t of the group, word w and code n of the lane in the 2-bit tile); columns through the rank position rule."""
    Mp, Kp = -(-M // 256) * 256, -(-K // 256) * 256
    strips, nkt = Mp // 16, Kp // 256
    U = np.zeros((M, K), dtype=np.int8)
    value = {0: 0, 1: 1, 2: -1}
    for r in range(M):
        strip, i = r // 16, r % 16
        G, t = strip // 5, strip % 5
        for c in range(K):
            pc = _rank_position(c, K)
            T, cc = pc // 256, pc % 256
            h, kk = cc >> 7, cc & 127
            g = ((kk >> 6) & 1) | (((kk >> 4) & 1) << 1)
            e = (((kk >> 5) & 1) << 4) | (kk & 15)
            v, n8 = e >> 3, e & 7
            lane, w, n = 16 * g + i, 2 * h + (v >> 1), 2 * n8 + (v & 1)
            q = 64 * t + 16 * w + n
            j, d = q // 5, q % 5
            byte = int(blob[(G * nkt + T) * 4096 + (j >> 4) * 1024 + lane * 16 + (j & 15)])
            U[r, c] = value[(byte // 3 ** d) % 3]
    return U


@pytest.mark.parametrize("M,K", [(1, 1), (17, 33), (80, 256), (81, 300), (200, 70), (96, 513)])
def test_dense_code_round_trip_and_position_rule(M, K):
    U = workloads.make_inputs(M, 8, K, 1, 0.6, 0.02, "f32", seed=M + 7 * K).U
    blob = tsvd.tsvd_dense_pack_host(U)
    assert blob.nbytes == tsvd.tsvd_dense_bytes(M, K)
    assert blob.max() <= 242
    assert np.array_equal(tsvd.tsvd_dense_unpack_host(blob, M, K), U)
    assert np.array_equal(_dense_decode(blob, M, K), U)
    assert np.array_equal(blob, tsvd.tsvd_dense_pack_host(U))


def test_dense_code_is_1_6_bits_per_element_and_rejects_corruption():
    assert tsvd.tsvd_dense_bytes(16384, 8192) * 8 == int(1.6 * 16400 * 8192)       # 205 groups of 80 rows: 16400 rows stored
    assert tsvd.tsvd_dense_bytes(16384, 8192) / (16384 * 8192 / 4) < 0.801           # against 2 bits per element
    U = workloads.make_inputs(40, 8, 300, 1, 0.5, 0.02, "f32", seed=3).U
    blob = tsvd.tsvd_dense_pack_host(U)
    bad = blob.copy()
    bad[5] = 250                                                                      # not a number below 3^5
    with pytest.raises(tsvd.TsvdError) as e:
        tsvd.tsvd_dense_unpack_host(bad, 40, 300)
    assert e.value.status == 2
    U2 = U.copy()
    U2[3, 3] = 2
    lib = tsvd.load_library()
    out = np.full(blob.nbytes, 0xAB, dtype=np.uint8)
    assert lib.tsvd_dense_pack_host(U2.ctypes.data, 40, 300, out.ctypes.data, out.nbytes) == 2 and np.all(out == 0xAB)
    assert lib.tsvd_dense_pack_host(U.ctypes.data, 40, 300, out.ctypes.data, out.nbytes - 1) == 1


def test_bench_reads_traffic_records_from_the_tracked_profile():
    """bench.py takes roofline.traffic from profiles/hbm_traffic_fetch_write_size.md and only for the kernel selection
    the record was measured on."""
    import bench
    got = bench._traffic_from_profile("opt66b_fc1_prefill", "tsvd_gemm_fp6_kernel:40")
    assert got is not None and 1.5e9 < got < 4e9
    assert bench._traffic_from_profile("opt66b_fc1_prefill", "tsvd_gemm_pipe_kernel:1") is None      # another kernel: no claim
    assert bench._traffic_from_profile("no_such_workload", "x") is None
