"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bars (from the benchmark spec):
  * activation codes bit-exact, else mismatch rate <= 1e-5 with off-by-one differences only;
  * int32 accumulators bit-exact given identical codes;
  * bf16 outputs: max rel err <= 1e-2 and mean rel err <= 1e-3, with
    rel = |y - y_ref| / max(|y_ref|, 1e-3 * rms(y_ref row)).
"""
import math

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import hbl_oracle as O
from paper_2504_18415_amd import synth

pytestmark = pytest.mark.gpu

EPS = 1e-5


def note(msg):
    """Name the case before each GPU step (survives a lost box: flushed line by line)."""
    print(f"[gpu-case] {msg}", flush=True)


@pytest.fixture(scope="module")
def hbl():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2504_18415_amd import hbl as H
    H.lib()
    return H


def dev_x(x_np):
    """numpy fp32 array or uint16 bf16 bit patterns -> device tensor of the matching torch dtype."""
    if x_np.dtype == np.uint16:
        return torch.from_numpy(x_np.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(x_np).cuda()


def host_bf16_bits(y):
    return y.view(torch.int16).cpu().numpy().view(np.uint16)


def rel_err(y_bits, ref_bits):
    y = synth.bf16_bits_to_f32(y_bits).astype(np.float64)
    r = synth.bf16_bits_to_f32(ref_bits).astype(np.float64)
    rms = np.sqrt((r ** 2).mean(axis=1, keepdims=True))
    den = np.maximum(np.abs(r), 1e-3 * rms + 1e-30)
    e = np.abs(y - r) / den
    return e.max(), e.mean()


def check_codes(got, want):
    diff = got.astype(np.int16) - want.astype(np.int16)
    bad = diff != 0
    rate = bad.mean()
    assert rate <= 1e-5, f"code mismatch rate {rate}"
    assert np.abs(diff).max(initial=0) <= 1
    return rate


_WEIGHT_CACHE = {}


def setup_weights(hbl, site):
    """Ternarise (oracle and GPU, per scale group) and pack the site's weights; cached per weight recipe."""
    key = (site.K, site.N, site.seed, site.w_stream, site.groups, site.w_std)
    if key not in _WEIGHT_CACHE:
        if len(_WEIGHT_CACHE) > 6:
            _WEIGHT_CACHE.clear()
        _WEIGHT_CACHE[key] = _setup_weights(hbl, site)
    return _WEIGHT_CACHE[key]


def _setup_weights(hbl, site):
    W = synth.make_w(site)
    wc_ref = np.empty((site.N, site.K), np.int8)
    alphas_ref = np.empty(site.groups, np.float32)
    rows = site.N // site.groups
    wc_dev, al_dev = [], []
    for g in range(site.groups):
        blk = np.ascontiguousarray(W[g * rows:(g + 1) * rows])
        c, a = O.ternarize_weights_absmean(blk, EPS)
        wc_ref[g * rows:(g + 1) * rows] = c
        alphas_ref[g] = a
        cd, ad = hbl.ternarize_weights_absmean(torch.from_numpy(blk).cuda(), EPS)
        wc_dev.append(cd)
        al_dev.append(ad)
    wc_d = torch.cat(wc_dev, 0).contiguous()
    al_d = torch.cat(al_dev).contiguous()
    packed = hbl.pack_ternary_2bit(wc_d)
    torch.cuda.synchronize()
    return wc_ref, alphas_ref, wc_d, al_d, packed


# ------------------------------------------------------------------ set-up kernels
@pytest.mark.parametrize("N,K", [(32, 128), (96, 384), (256, 256), (320, 2048)])
def test_ternarize_and_pack_roundtrip(hbl, N, K):
    note(f"ternarize/pack N={N} K={K}")
    site = synth.Site("w", 1, K, N, seed=20 + N)
    W = synth.make_w(site)
    c_ref, a_ref = O.ternarize_weights_absmean(W, EPS)
    c_dev, a_dev = hbl.ternarize_weights_absmean(torch.from_numpy(W).cuda(), EPS)
    assert a_dev.cpu().numpy()[0] == a_ref
    assert np.array_equal(c_dev.cpu().numpy(), c_ref)
    packed = hbl.pack_ternary_2bit(c_dev)
    assert packed.numel() == hbl.packed_bytes(N, K)
    row_sums = packed[N * K // 4:N * K // 4 + 4 * N].view(torch.int32).cpu().numpy()
    assert np.array_equal(row_sums, c_ref.astype(np.int32).sum(1))
    back = hbl.unpack_ternary_2bit(packed, N, K)
    assert np.array_equal(back.cpu().numpy(), c_ref)


def test_ternarize_odd_sizes_and_scale(hbl):
    note("ternarize odd sizes")
    rng = np.random.default_rng(5)
    for shape, std in [((7, 13), 1.0), ((1, 1), 0.3), ((129, 1000), 1e-3), ((3, 70000), 5.0)]:
        W = (rng.standard_normal(shape) * std).astype(np.float32)
        c_ref, a_ref = O.ternarize_weights_absmean(W, EPS)
        c_dev, a_dev = hbl.ternarize_weights_absmean(torch.from_numpy(W).cuda(), EPS)
        assert a_dev.cpu().numpy()[0] == a_ref, shape
        assert np.array_equal(c_dev.cpu().numpy(), c_ref), shape


# ------------------------------------------------------------------ activation front end
ALL_K = [128, 256, 512, 1024, 2048, 4096, 8192, 16384]


@pytest.mark.parametrize("K", ALL_K)
def test_fwht_exact_integers_on_gpu(hbl, K):
    """Small-integer rows make every butterfly exact, so INT8 codes of H x are fixed by integer
    arithmetic alone (no dependence on stage order): a pure check of the butterfly network."""
    note(f"fwht exact integers K={K}")
    rng = np.random.default_rng(K)
    x = rng.integers(-3, 4, size=(5, K)).astype(np.float32)
    codes, sd, cs = hbl.fwht_quant(torch.from_numpy(x).cuda(), 8, True, EPS)
    c_ref, s_ref, xr = O.fwht_quant(x, 8, hadamard=True, eps=EPS, want_xr=True)
    assert np.array_equal(codes.cpu().numpy(), c_ref)
    assert np.array_equal(sd.cpu().numpy(), s_ref)
    assert np.array_equal(cs.cpu().numpy(), c_ref.astype(np.int32).sum(1))
    # unit vectors: row j of H, all entries +-1/sqrt(K) -> every code is +-127
    e = np.zeros((2, K), np.float32)
    e[0, 1] = 1.0
    e[1, K - 1] = -2.0
    codes, _, _ = hbl.fwht_quant(torch.from_numpy(e).cuda(), 8, True, EPS)
    j = np.arange(K)
    sign0 = np.array([(-1) ** bin(int(v) & 1).count("1") for v in j])
    sign1 = -np.array([(-1) ** bin(int(v) & (K - 1)).count("1") for v in j])
    assert np.array_equal(np.sign(codes.cpu().numpy()[0]), sign0)
    assert np.array_equal(np.sign(codes.cpu().numpy()[1]), sign1)


@pytest.mark.parametrize("K", ALL_K)
@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("hadamard", [True, False])
def test_fwht_quant_parity(hbl, K, bits, hadamard):
    T = 37 if K <= 4096 else 19                       # ragged, several rows per wave-group
    for dtype in (synth.BF16, synth.F32):
        note(f"fwht_quant K={K} bits={bits} hadamard={hadamard} dtype={dtype} T={T}")
        site = synth.Site("a", T, K, 32, x_dtype=dtype, outlier_frac=0.01, outlier_scale=30.0, seed=K + bits)
        x = synth.make_x(site)
        c_ref, s_ref = O.fwht_quant(x, bits, hadamard=hadamard, eps=EPS)
        codes, sd, cs = hbl.fwht_quant(dev_x(x), bits, hadamard, EPS)
        assert np.array_equal(sd.cpu().numpy(), s_ref)
        rate = check_codes(codes.cpu().numpy(), c_ref)
        assert rate == 0.0
        assert np.array_equal(cs.cpu().numpy(), c_ref.astype(np.int32).sum(1))


@pytest.mark.parametrize("K,hadamard", [(256, True), (4096, True), (16384, True), (640, False)])
def test_int4_offset_codes_and_split_calls(hbl, K, hadamard):
    """The forward calls carry INT4 codes as code+8 (bytes 0..15); the stage-level calls expose that form.
    Stored bytes must be oracle code + 8, the code sum the true sum, and the two-launch split must
    reproduce the single call bit for bit."""
    note(f"int4 offset codes K={K} hadamard={hadamard}")
    site = synth.Site("a", 45, K, 96, hadamard=hadamard, outlier_frac=0.01, outlier_scale=30.0, seed=K + 1)
    x = synth.make_x(site)
    c_ref, s_ref = O.fwht_quant(x, 4, hadamard=hadamard, eps=EPS)
    xd = dev_x(x)
    codes, sd, cs = hbl.fwht_quant(xd, 4, hadamard, EPS, code_offset=8)
    got = codes.cpu().numpy()
    assert got.min() >= 0 and got.max() <= 15
    assert np.array_equal(got, c_ref + 8)
    assert np.array_equal(cs.cpu().numpy(), c_ref.astype(np.int32).sum(1))
    assert np.array_equal(sd.cpu().numpy(), s_ref)
    wc_ref, al_ref, wc_d, al_d, packed = setup_weights(hbl, site)
    y_split = hbl.gemm_dequant_bf16(codes, sd, cs, packed, site.N, al_d, code_offset=8)
    codes0, sd0, cs0 = hbl.fwht_quant(xd, 4, hadamard, EPS, code_offset=0)
    y_split0 = hbl.gemm_dequant_bf16(codes0, sd0, cs0, packed, site.N, al_d, code_offset=0)
    fn = hbl.hbitlinear_forward if hadamard else hbl.plain_bitlinear_forward
    y_one = fn(xd, packed, site.N, al_d, 4, EPS)
    y_ref = O.bitlinear_forward(x, wc_ref, al_ref, 4, hadamard, EPS)
    assert np.array_equal(host_bf16_bits(y_split), host_bf16_bits(y_one))
    assert np.array_equal(host_bf16_bits(y_split0), host_bf16_bits(y_one))
    assert np.array_equal(host_bf16_bits(y_one), y_ref)
    with pytest.raises(hbl.HblError):
        hbl.fwht_quant(xd, 8, hadamard, EPS, code_offset=8)


def _record_image_words(T, K):
    """Index arithmetic of the record image (HBL_CODES_BF6), restated from its description: for token t and
    record m (features [32m, 32m+32)) the positions, in 8-byte words of the image, of the record's bits 0..63,
    64..127 and 128..191.  Tokens in panels of 128, features in blocks of 128, a block = 128 rows of 96 bytes."""
    t = np.arange(T, dtype=np.int64)[:, None]
    m = np.arange(K // 32, dtype=np.int64)[None, :]
    kb, s, h = m >> 2, (m >> 1) & 1, m & 1
    r = t & 127
    row = (((t >> 7) * (K // 128)) + kb) * 12288 + r * 96
    lo = row + (((3 * s + 2 * h) ^ ((r >> 3) & 1)) << 4)
    hi = row + (((3 * s + 1) ^ ((r >> 3) & 1)) << 4) + ((h ^ ((r >> 4) & 1)) << 3)
    return lo // 8, lo // 8 + 1, hi // 8


def record_image_bytes(T, K):
    return ((T + 127) // 128) * (K // 128) * 12288


def decode_bf6_records(image, T, K):
    """Record image bytes -> int codes [T, K]: per 32 features a 192-bit record of six-bit e3m2 floats, feature i
    at bits [6i, 6i+6)."""
    img = np.ascontiguousarray(image).view(np.uint8).reshape(-1)[:record_image_bytes(T, K)].view(np.uint64)
    w0, w1, w2 = _record_image_words(T, K)
    words = (img[w0], img[w1], img[w2])
    out = np.empty((T, K // 32, 32), np.int32)
    for i in range(32):
        word, off = divmod(6 * i, 64)
        v = (words[word] >> np.uint64(off)) & np.uint64(0x3F)
        if off > 58:
            v |= (words[word + 1] << np.uint64(64 - off)) & np.uint64(0x3F)
        v = v.astype(np.int32)
        sign, e, mant = v >> 5, (v >> 2) & 7, v & 3
        mag = np.where(e == 0, mant / 16.0, (2.0 ** (e - 3)) * (1 + mant / 4.0))
        val = np.where(sign == 1, -mag, mag)
        out[:, :, i] = val.astype(np.int32)
        assert np.all(val == out[:, :, i])       # every stored value is an integer
    return out.reshape(T, K)


def record_bits(image, T, K):
    """The 192 bits of every record as three uint64 words [T, K/32, 3] (what a comparison bit for bit looks at:
    the image also holds rows beyond T that nobody wrote)."""
    img = np.ascontiguousarray(image).view(np.uint8).reshape(-1)[:record_image_bytes(T, K)].view(np.uint64)
    w0, w1, w2 = _record_image_words(T, K)
    return np.stack([img[w0], img[w1], img[w2]], axis=-1)


@pytest.mark.parametrize("K,hadamard", [(4096, True), (8192, True), (16384, True), (512, True), (1024, True),
                                        (2048, True), (2048, False), (4096, False), (16384, False),
                                        (640, False), (1536, False), (11008, False)])
def test_bf6_code_records_and_f6f4_gemm(hbl, K, hadamard):
    """INT4 codes as 6-bit float records (the form the fp6 x fp4 matrix-core path reads), from every
    quantiser kernel that writes them: the decoded records equal the oracle codes, and the two-launch
    split on that path reproduces the oracle's outputs and the int8 path bit for bit."""
    note(f"bf6 records K={K} hadamard={hadamard}")
    T, N = 150, 288
    site = synth.Site("a", T, K, N, hadamard=hadamard, outlier_frac=0.01, outlier_scale=30.0, seed=K + 6)
    x = synth.make_x(site)
    c_ref, s_ref = O.fwht_quant(x, 4, hadamard=hadamard, eps=EPS)
    xd = dev_x(x)
    rec, sd, cs = hbl.fwht_quant(xd, 4, hadamard, EPS, code_offset=hbl.CODES_BF6)
    rec_np = rec.cpu().numpy().view(np.uint8)
    assert rec_np.size == record_image_bytes(T, K) == hbl.code_bytes(T, K, hbl.CODES_BF6)
    assert np.array_equal(decode_bf6_records(rec_np, T, K), c_ref.astype(np.int32))
    # and bit for bit: every record holds the canonical patterns (code 0 is +0, never -0)
    want = encode_bf6_records(c_ref.astype(np.int32))
    assert np.array_equal(record_bits(rec_np, T, K), record_bits(want, T, K))
    assert np.array_equal(sd.cpu().numpy(), s_ref)
    assert np.array_equal(cs.cpu().numpy(), c_ref.astype(np.int32).sum(1))
    wc_ref, al_ref, wc_d, al_d, packed = setup_weights(hbl, site)
    y6 = hbl.gemm_dequant_bf16(rec, sd, cs, packed, N, al_d, code_offset=hbl.CODES_BF6, K=K)
    c8, sd8, cs8 = hbl.fwht_quant(xd, 4, hadamard, EPS, code_offset=8)
    y8 = hbl.gemm_dequant_bf16(c8, sd8, cs8, packed, N, al_d, code_offset=8)
    fn = hbl.hbitlinear_forward if hadamard else hbl.plain_bitlinear_forward
    y1 = fn(xd, packed, N, al_d, 4, EPS)
    y_ref = O.bitlinear_forward(x, wc_ref, al_ref, 4, hadamard, EPS)
    assert np.array_equal(host_bf16_bits(y6), y_ref)
    assert np.array_equal(host_bf16_bits(y8), y_ref)
    assert np.array_equal(host_bf16_bits(y1), y_ref)
    # records need 8-element chunks per lane: rows shorter than 512 and INT8 codes are rejected
    with pytest.raises(hbl.HblError):
        hbl.fwht_quant(xd[:, :256].contiguous(), 4, hadamard, EPS, code_offset=hbl.CODES_BF6)
    with pytest.raises(hbl.HblError):
        hbl.fwht_quant(xd, 8, hadamard, EPS, code_offset=hbl.CODES_BF6)


BF6_OF_CODE = {-8: 0x38, -7: 0x37, -6: 0x36, -5: 0x35, -4: 0x34, -3: 0x32, -2: 0x30, -1: 0x2C, 0: 0x00,
               1: 0x0C, 2: 0x10, 3: 0x12, 4: 0x14, 5: 0x15, 6: 0x16, 7: 0x17}


def encode_bf6_records(codes):
    """int codes [T, K] in [-8, 7] -> record image bytes (inverse of decode_bf6_records; rows of the last
    panel beyond T are zero)."""
    T, K = codes.shape
    lut = np.zeros(16, np.uint64)
    for c, v in BF6_OF_CODE.items():
        lut[c + 8] = v
    six = lut[codes.astype(np.int64) + 8].reshape(T, K // 32, 32)
    words = [np.zeros((T, K // 32), np.uint64) for _ in range(3)]
    for i in range(32):
        word, off = divmod(6 * i, 64)
        words[word] |= (six[:, :, i] << np.uint64(off))
        if off > 58:
            words[word + 1] |= six[:, :, i] >> np.uint64(64 - off)
    img = np.zeros(record_image_bytes(T, K) // 8, np.uint64)
    w0, w1, w2 = _record_image_words(T, K)
    img[w0], img[w1], img[w2] = words[0], words[1], words[2]
    return img.view(np.uint8)


@pytest.mark.parametrize("K,T", [(16384, 1100), (8192, 2300), (4096, 4500)])
def test_quantiser_rows_walked_by_resident_workgroups(hbl, K, T):
    """More rows than the chip holds workgroups of the K >= 4096 quantiser at once: every workgroup then walks
    several rows (the last round ragged), loading the next row while it finishes the current one.  Codes, scales
    and code sums of all rows against the oracle, in the record form and both byte forms."""
    note(f"row-walking quantiser K={K} T={T}")
    site = synth.Site("a", T, K, 32, hadamard=True, outlier_frac=0.01, outlier_scale=30.0, seed=K + T)
    x = synth.make_x(site)
    xd = dev_x(x)
    c4, s4 = O.fwht_quant(x, 4, hadamard=True, eps=EPS)
    rec, sd, cs = hbl.fwht_quant(xd, 4, True, EPS, code_offset=hbl.CODES_BF6)
    want = record_bits(encode_bf6_records(c4.astype(np.int32)), T, K)
    assert np.array_equal(record_bits(rec.cpu().numpy(), T, K), want)
    assert np.array_equal(sd.cpu().numpy(), s4)
    assert np.array_equal(cs.cpu().numpy(), c4.astype(np.int32).sum(1))
    c, sd, cs = hbl.fwht_quant(xd, 4, True, EPS, code_offset=8)
    assert np.array_equal(c.cpu().numpy().astype(np.int32) - 8, c4.astype(np.int32))
    assert np.array_equal(sd.cpu().numpy(), s4) and np.array_equal(cs.cpu().numpy(), c4.astype(np.int32).sum(1))
    c8, s8 = O.fwht_quant(x, 8, hadamard=True, eps=EPS)
    c, sd, cs = hbl.fwht_quant(xd, 8, True, EPS)
    assert np.array_equal(c.cpu().numpy(), c8)
    assert np.array_equal(sd.cpu().numpy(), s8) and np.array_equal(cs.cpu().numpy(), c8.astype(np.int32).sum(1))


def test_f6f4_gemm_extreme_codes(hbl):
    """Hand-made records: every code -8 (one row +7, one row random) against all-(+1) / all-(-1) weight
    rows - the largest accumulator magnitude the path can see (8 * 16384 = 2^17) must come out exact
    from the fp32 accumulators of the fp6 x fp4 matrix cores."""
    note("f6f4 extreme codes")
    T, K, N = 130, 16384, 64
    rng = np.random.default_rng(9)
    codes = np.full((T, K), -8, np.int8)
    codes[7] = 7
    codes[9] = rng.integers(-8, 8, K)
    assert np.array_equal(decode_bf6_records(encode_bf6_records(codes), T, K), codes)
    wc = np.ones((N, K), np.int8)
    wc[1::2] = -1
    wc[5] = rng.integers(-1, 2, K)
    packed = hbl.pack_ternary_2bit(torch.from_numpy(wc).cuda())
    al = torch.ones(1, dtype=torch.float32, device="cuda")
    sd = torch.ones(T, dtype=torch.float32, device="cuda")
    cs = torch.from_numpy(codes.astype(np.int32).sum(1).astype(np.int32)).cuda()
    rec = torch.from_numpy(encode_bf6_records(codes).view(np.int8)).cuda()
    y = hbl.gemm_dequant_bf16(rec, sd, cs, packed, N, al, code_offset=hbl.CODES_BF6, K=K)
    acc = O.gemm_i32(codes, wc)
    assert np.abs(acc).max() == 8 * K
    want = O.dequant_bf16(acc, np.ones(T, np.float32), np.ones(1, np.float32))
    assert np.array_equal(host_bf16_bits(y), want)
    # rows whose sums are exactly representable in bf16 pin the integers themselves
    assert synth.bf16_bits_to_f32(host_bf16_bits(y))[0, 0] == -8.0 * K
    assert synth.bf16_bits_to_f32(host_bf16_bits(y))[7, 1] == -7.0 * K


@pytest.mark.parametrize("K", [384, 1536, 11008 // 128 * 128])
def test_plain_quant_non_power_of_two(hbl, K):
    note(f"plain quant K={K}")
    site = synth.Site("a", 9, K, 32, outlier_frac=0.01, outlier_scale=30.0, seed=K)
    x = synth.make_x(site)
    for bits in (4, 8):
        c_ref, s_ref = O.fwht_quant(x, bits, hadamard=False, eps=EPS)
        codes, sd, cs = hbl.fwht_quant(dev_x(x), bits, False, EPS)
        assert np.array_equal(codes.cpu().numpy(), c_ref)
        assert np.array_equal(sd.cpu().numpy(), s_ref)
        assert np.array_equal(cs.cpu().numpy(), c_ref.astype(np.int32).sum(1))


def test_zero_rows_and_single_token(hbl):
    note("zero rows")
    x = np.zeros((3, 512), np.float32)
    x[1, 7] = 4.0
    for bits in (4, 8):
        codes, sd, cs = hbl.fwht_quant(torch.from_numpy(x).cuda(), bits, True, EPS)
        c_ref, s_ref = O.fwht_quant(x, bits, hadamard=True, eps=EPS)
        assert np.array_equal(codes.cpu().numpy(), c_ref) and np.array_equal(sd.cpu().numpy(), s_ref)
        assert not codes.cpu().numpy()[0].any() and sd.cpu().numpy()[0] == 0


# ------------------------------------------------------------------ integer GEMM
@pytest.mark.parametrize("T,K,N", [
    (1, 128, 32), (5, 256, 96), (31, 384, 288), (33, 512, 544), (64, 2048, 256), (65, 1024, 320),
    (130, 640, 416), (257, 2048, 512), (300, 4096, 288), (1000, 256, 1056),
])
def test_gemm_i32_bit_exact(hbl, T, K, N):
    note(f"gemm_i32 T={T} K={K} N={N}")
    rng = np.random.default_rng(T * 7 + N)
    q = rng.integers(-128, 128, (T, K)).astype(np.int8)
    c = rng.integers(-1, 2, (N, K)).astype(np.int8)
    packed = hbl.pack_ternary_2bit(torch.from_numpy(c).cuda())
    acc = hbl.gemm_i32(torch.from_numpy(q).cuda(), packed, N)
    assert np.array_equal(acc.cpu().numpy(), O.gemm_i32(q, c))


def test_gemm_i32_one_hot_layout(hbl):
    """One-hot operands: acc[t][o] = q[t][k0]*c[o][k0]; catches any row/column/K permutation mistake."""
    note("gemm_i32 one-hot")
    T, K, N = 70, 512, 96
    for k0 in (0, 17, 130, 511):
        q = np.zeros((T, K), np.int8)
        c = np.zeros((N, K), np.int8)
        q[:, k0] = (np.arange(T) % 250 - 125).astype(np.int8)
        c[:, k0] = (np.arange(N) % 3 - 1).astype(np.int8)
        packed = hbl.pack_ternary_2bit(torch.from_numpy(c).cuda())
        acc = hbl.gemm_i32(torch.from_numpy(q).cuda(), packed, N).cpu().numpy()
        assert np.array_equal(acc, np.outer(q[:, k0].astype(np.int32), c[:, k0].astype(np.int32)))


# ------------------------------------------------------------------ end to end
def run_site(hbl, site, bits, sample_rows=None):
    """Runs one projection on the GPU and the oracle; returns the comparison figures."""
    x = synth.make_x(site)
    wc_ref, al_ref, wc_d, al_d, packed = setup_weights(hbl, site)
    assert np.array_equal(al_d.cpu().numpy(), al_ref)
    assert np.array_equal(wc_d.cpu().numpy(), wc_ref)
    xd = dev_x(x)
    fn = hbl.hbitlinear_forward if site.hadamard else hbl.plain_bitlinear_forward
    y = fn(xd, packed, site.N, al_d, bits, EPS)
    codes, sd, cs = hbl.fwht_quant(xd, bits, site.hadamard, EPS)
    acc = hbl.gemm_i32(codes, packed, site.N)
    # the forward call above ran the fp6 x fp4 kernel if INT4, T > 64, K >= 512: that kernel's own accumulators,
    # from the code records it reads, in the launch configuration the forward call takes for this shape
    acc6 = None
    if bits == 4 and site.T > 64 and site.K >= 512:
        rec, _, _ = hbl.fwht_quant(xd, 4, site.hadamard, EPS, code_offset=hbl.CODES_BF6)
        acc6 = hbl.gemm_i32_bf6(rec, packed, site.N, site.T, site.K)
        del rec
    torch.cuda.synchronize()
    rows = np.arange(site.T) if sample_rows is None else sample_rows
    xs = np.ascontiguousarray(x[rows])
    y_ref, c_ref, s_ref, a_ref = O.bitlinear_forward(xs, wc_ref, al_ref, bits, site.hadamard, EPS,
                                                     want_intermediates=True)
    rows_t = torch.from_numpy(rows).cuda()
    c_got = codes[rows_t].cpu().numpy()
    rate = check_codes(c_got, c_ref)
    assert np.array_equal(sd[rows_t].cpu().numpy(), s_ref)
    same = (c_got == c_ref).all(axis=1)
    a_got = acc[rows_t].cpu().numpy()
    assert np.array_equal(a_got[same], a_ref[same]), "int32 accumulators differ on rows with identical codes"
    if acc6 is not None:
        a6 = acc6[rows_t].cpu().numpy()
        assert np.array_equal(a6[same], a_ref[same]), "fp6 x fp4 kernel: accumulators differ from the int32 contraction"
    y_bits = host_bf16_bits(y[rows_t])
    mx, mean = rel_err(y_bits, y_ref)
    assert mx <= 1e-2 and mean <= 1e-3, (mx, mean)
    exact = float((y_bits == y_ref).mean())
    note(f"   {site.name} bits={bits}: code mismatch {rate:.2e}, y bit-exact {exact:.6f}, max rel {mx:.2e}")
    return rate, exact


def test_config1_tiny(hbl):
    note("config 1")
    rate, exact = run_site(hbl, synth.config_sites(1)[0], 4)
    assert rate == 0 and exact == 1.0


@pytest.mark.parametrize("bits", [4, 8])
def test_config2_wo_1p3b(hbl, bits):
    note(f"config 2 bits={bits}")
    run_site(hbl, synth.config_sites(2)[0], bits)


@pytest.mark.parametrize("T,K,N", [(96, 8192, 320), (200, 16384, 96), (77, 4096, 544)])
def test_configs_3_4_reduced_shapes(hbl, T, K, N):
    """Same recipes as configs 3 and 4 at sizes the oracle finishes in seconds (several tiles, ragged T)."""
    note(f"reduced cfg3/4 T={T} K={K} N={N}")
    run_site(hbl, synth.shrink(synth.config_sites(3)[0], T=T, K=K, N=N), 4)
    run_site(hbl, synth.shrink(synth.config_sites(4)[1], T=T, K=K, N=N), 4)


@pytest.mark.parametrize("T,K,N", [(300, 16384, 1056), (130, 8192, 2048), (513, 16384, 416)])
def test_mid_size_batch_split_k(hbl, T, K, N):
    """Between 65 tokens and about a thousand a long-K projection has few output tiles: the fp6 x fp4 GEMM then
    splits K over workgroups and a reduction launch adds the int32 partial tiles.  Ragged T and N, splits of 8, 4
    and 2; every output against the oracle."""
    note(f"mid-size batch split-K T={T} K={K} N={N}")
    run_site(hbl, synth.shrink(synth.config_sites(4)[1], T=T, K=K, N=N), 4)
    run_site(hbl, synth.shrink(synth.config_sites(4)[1], T=T, K=K, N=N), 8)     # the int8 kernel's split form


def panel_rows(T, seed, panel=128):
    """First and last token row of every `panel`-token workgroup panel of the prefill GEMM launch, plus one
    seeded row inside each: every workgroup row of the launch has rows under the oracle."""
    rng = np.random.default_rng(seed)
    rows = []
    for p0 in range(0, T, panel):
        p1 = min(p0 + panel, T) - 1
        rows += [p0, p1, int(rng.integers(p0, p1 + 1))]
    return np.unique(np.asarray(rows, dtype=np.int64))


def test_config3_full_size_sampled(hbl):
    note("config 3 full size, rows of every token panel")
    site = synth.config_sites(3)[0]
    rate, exact = run_site(hbl, site, 4, sample_rows=panel_rows(site.T, 3))
    assert rate == 0 and exact == 1.0


@pytest.mark.parametrize("idx", [0, 1])
def test_config4_full_size_sampled(hbl, idx):
    """7B prefill sites in the launch configuration the benchmark times; the oracle on the first, the last and
    one more token row of every 128-token workgroup panel (all 64 of them), every output of those rows and
    the timed kernel's own int32 accumulators bit for bit."""
    site = synth.config_sites(4)[idx]
    note(f"config 4 {site.name} full size, rows of every token panel")
    rate, exact = run_site(hbl, site, 4, sample_rows=panel_rows(site.T, 4 + idx))
    assert rate == 0 and exact == 1.0


def test_config4_wdown_swiglu_input(hbl):
    """Configuration 4's W_down with its input drawn as a gated-activation output SiLU(a)*b (heavy-tailed,
    mostly small values) and the same 1 % outlier channels x50: parity-only variant of the site above."""
    site = synth.config4_wdown_swiglu()
    note("config 4 wdown_7b, SwiGLU-shaped input, rows of every token panel")
    rate, exact = run_site(hbl, site, 4, sample_rows=panel_rows(site.T, 44))
    assert rate == 0 and exact == 1.0
    run_site(hbl, synth.shrink(site, T=200, N=96), 4)            # and every row of a reduced shape


@pytest.mark.parametrize("T,K,N", [(300, 1024, 544), (129, 4096, 96), (513, 512, 1056)])
def test_prefill_gemm_tiles_raw_accumulators(hbl, T, K, N):
    """Every workgroup tile of both prefill GEMM kernels (256 x 256, 128 x 128, 512 x 128, and the fp6 x fp4
    kernel's K cut over workgroups) on ragged shapes: the int32 accumulators, read straight out of the
    kernel, against the oracle's integer contraction - every element, bit for bit."""
    note(f"prefill GEMM tiles, raw accumulators T={T} K={K} N={N}")
    rng = np.random.default_rng(T + K + N)
    q = rng.integers(-8, 8, (T, K)).astype(np.int8)
    q[3] = -8                                                     # the largest magnitudes the codes can take
    q[5] = 7
    c = rng.integers(-1, 2, (N, K)).astype(np.int8)
    c[1] = 1
    c[2] = -1
    want = O.gemm_i32(q, c)
    packed = hbl.pack_ternary_2bit(torch.from_numpy(c).cuda())
    rec = torch.from_numpy(encode_bf6_records(q.astype(np.int32)).view(np.int8)).cuda()
    qd = torch.from_numpy(q).cuda()
    for tile in (hbl.TILE_SQUARE, hbl.TILE_SMALL, hbl.TILE_WIDE, hbl.TILE_SPLIT_K):
        got = hbl.gemm_i32_tile_for_tests(rec, hbl.CODES_BF6, packed, N, tile, T=T, K=K).cpu().numpy()
        assert np.array_equal(got, want), f"fp6 x fp4 kernel, tile {tile}"
    q8 = rng.integers(-128, 128, (T, K)).astype(np.int8)
    want8 = O.gemm_i32(q8, c)
    q8d = torch.from_numpy(q8).cuda()
    for tile in (hbl.TILE_SQUARE, hbl.TILE_SMALL, hbl.TILE_WIDE):
        got = hbl.gemm_i32_tile_for_tests(q8d, hbl.CODES_INT8, packed, N, tile).cpu().numpy()
        assert np.array_equal(got, want8), f"int8 kernel, tile {tile}"
        got = hbl.gemm_i32_tile_for_tests(qd, hbl.CODES_INT8, packed, N, tile).cpu().numpy()
        assert np.array_equal(got, want), f"int8 kernel on INT4 codes, tile {tile}"
    assert np.array_equal(hbl.gemm_i32_bf6(rec, packed, N, T, K).cpu().numpy(), want)      # the forward's own choice


def test_f6f4_raw_accumulators_extreme_and_split_k_shapes(hbl):
    """|acc| = 8 * 16384 = 2^17 out of the fp6 x fp4 kernel as an integer, and the mid-size-batch shapes on
    which the forward call itself cuts K (8, 4 and 2 slices): raw accumulators against the oracle."""
    note("f6f4 raw accumulators: extremes and the forward's own K cuts")
    rng = np.random.default_rng(17)
    for T, K, N in [(130, 16384, 64), (300, 16384, 1056), (130, 8192, 2048), (513, 16384, 416)]:
        q = rng.integers(-8, 8, (T, K)).astype(np.int8)
        q[0] = -8
        q[T - 1] = 7
        c = rng.integers(-1, 2, (N, K)).astype(np.int8)
        c[0] = 1
        c[N - 1] = -1
        want = O.gemm_i32(q, c)
        assert np.abs(want).max() == 8 * K
        packed = hbl.pack_ternary_2bit(torch.from_numpy(c).cuda())
        rec = torch.from_numpy(encode_bf6_records(q.astype(np.int32)).view(np.int8)).cuda()
        assert np.array_equal(hbl.gemm_i32_bf6(rec, packed, N, T, K).cpu().numpy(), want), (T, K, N)
        got = hbl.gemm_i32_tile_for_tests(rec, hbl.CODES_BF6, packed, N, hbl.TILE_SPLIT_K, T=T, K=K).cpu().numpy()
        assert np.array_equal(got, want), (T, K, N, "split-K tile")


@pytest.mark.parametrize("T,K,N,groups,bits,hadamard", [
    (1, 512, 32, 1, 4, True), (7, 2048, 96, 3, 4, False), (33, 4096, 544, 1, 8, True), (64, 1024, 160, 1, 4, True),
    (17, 8192, 288, 1, 4, True), (64, 640, 96, 1, 8, False), (5, 16384, 64, 2, 4, True),
])
def test_small_batch_split_k_path(hbl, T, K, N, groups, bits, hadamard):
    """T <= 64 takes the split-K kernel pair (partial tiles + reduction): ragged T, N not a multiple of the
    128-row workgroup tile, several scale groups, both code widths."""
    note(f"split-K T={T} K={K} N={N} groups={groups} bits={bits} hadamard={hadamard}")
    site = synth.Site("s", T, K, N, hadamard=hadamard, groups=groups, outlier_frac=0.01, outlier_scale=30.0,
                      seed=T + K + N)
    rate, exact = run_site(hbl, site, bits)
    assert rate == 0 and exact == 1.0


@pytest.mark.parametrize("batch", [1, 8, 32, 64])
def test_config5_decode_layer(hbl, batch):
    note(f"config 5 batch={batch}")
    for site in synth.config_sites(5, batch=batch):
        run_site(hbl, site, 4)


def test_forward_reuses_caller_buffers_and_is_deterministic(hbl):
    note("determinism / caller buffers")
    site = synth.shrink(synth.config_sites(2)[0], T=300, K=1024, N=288)
    x = dev_x(synth.make_x(site))
    _, _, _, al_d, packed = setup_weights(hbl, site)
    ws = hbl.alloc_workspace(site.T, site.K, site.N, 4)
    y1 = torch.empty((site.T, site.N), dtype=torch.bfloat16, device="cuda")
    y2 = torch.empty_like(y1)
    hbl.hbitlinear_forward(x, packed, site.N, al_d, 4, EPS, y=y1, workspace=ws)
    hbl.hbitlinear_forward(x, packed, site.N, al_d, 4, EPS, y=y2, workspace=ws)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        y3 = hbl.hbitlinear_forward(x, packed, site.N, al_d, 4, EPS)
    s.synchronize()
    torch.cuda.synchronize()
    assert torch.equal(y1.view(torch.int16), y2.view(torch.int16))
    assert torch.equal(y1.view(torch.int16), y3.view(torch.int16))


def test_empty_batch_and_errors_on_device(hbl):
    note("empty batch / errors")
    x = torch.empty((0, 256), dtype=torch.bfloat16, device="cuda")
    packed = torch.zeros(hbl.packed_bytes(256, 256), dtype=torch.uint8, device="cuda")
    al = torch.ones(1, dtype=torch.float32, device="cuda")
    y = hbl.hbitlinear_forward(x, packed, 256, al, 4)
    assert y.shape == (0, 256)
    with pytest.raises(hbl.HblError) as e:
        hbl.hbitlinear_forward(torch.zeros((4, 192), dtype=torch.bfloat16, device="cuda"), packed, 256, al, 4)
    assert e.value.status == hbl.E_SHAPE
    with pytest.raises(hbl.HblError) as e:
        hbl.hbitlinear_forward(torch.zeros((4, 256), dtype=torch.bfloat16, device="cuda"), packed, 256, al, 6)
    assert e.value.status == hbl.E_BITS


def run_group(hbl, sites, bits_list, expect_exact=True):
    """One grouped call over `sites` against the oracle, problem by problem, and against the
    stand-alone forward calls (must be bit-identical)."""
    items, refs, singles = [], [], []
    for site, bits in zip(sites, bits_list):
        x = synth.make_x(site)
        wc_ref, al_ref, wc_d, al_d, packed = setup_weights(hbl, site)
        xd = dev_x(x)
        items.append((xd, packed, site.N, al_d, bits, site.hadamard, None))
        refs.append(O.bitlinear_forward(x, wc_ref, al_ref, bits, site.hadamard, EPS) if site.T else None)
        fn = hbl.hbitlinear_forward if site.hadamard else hbl.plain_bitlinear_forward
        singles.append(fn(xd, packed, site.N, al_d, bits, EPS))
    ys = hbl.bitlinear_forward_grouped(items, EPS)
    torch.cuda.synchronize()
    for site, y, ref, single in zip(sites, ys, refs, singles):
        assert y.shape == (site.T, site.N)
        if site.T == 0:
            continue
        got = host_bf16_bits(y)
        assert np.array_equal(got, host_bf16_bits(single)), f"{site.name}: grouped differs from the single call"
        if expect_exact:
            assert np.array_equal(got, ref), f"{site.name}: grouped differs from the oracle"
        else:
            mx, mean = rel_err(got, ref)
            assert mx <= 1e-2 and mean <= 1e-3, (site.name, mx, mean)


@pytest.mark.parametrize("batch", [1, 8, 16, 32, 64])
def test_grouped_config5_decode_layer(hbl, batch):
    """The four projections of the 7B decode layer in one grouped call."""
    note(f"grouped config 5 batch={batch}")
    sites = synth.config_sites(5, batch=batch)
    run_group(hbl, sites, [4] * len(sites), expect_exact=False)


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("x_dtype", [synth.BF16, synth.F32])
def test_grouped_ragged_mix(hbl, bits, x_dtype):
    """Mixed token counts, row counts that are no multiple of 128, a row length that is no power of
    two, every Hadamard kernel family, an empty problem and scale groups - both small-batch forms."""
    note(f"grouped ragged bits={bits} dtype={x_dtype}")
    common = dict(outlier_frac=0.01, outlier_scale=30.0, x_dtype=x_dtype)
    for tmax in (3, 13, 29, 64):
        sites = [
            synth.Site("g_plain640", tmax, 640, 96, hadamard=False, seed=31, **common),
            synth.Site("g_h256", 1, 256, 32, hadamard=True, seed=32, **common),
            synth.Site("g_h2048", max(tmax - 2, 1), 2048, 288, hadamard=True, seed=33, groups=3, **common),
            synth.Site("g_empty", 0, 512, 64, hadamard=True, seed=34, **common),
            synth.Site("g_h8192", tmax, 8192, 160, hadamard=True, seed=35, **common),
            synth.Site("g_plain4096", 2, 4096, 544, hadamard=False, seed=36, **common),
            synth.Site("g_h16384", tmax, 16384, 64, hadamard=True, seed=37, **common),
        ]
        run_group(hbl, sites, [bits] * len(sites))


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("T", [33, 48, 64])
def test_grouped_two_token_tiles_short_and_odd_k(hbl, bits, T):
    """33-64 tokens take the shared form with two token tiles, which waits and synchronises once per two
    K-blocks and, on the fp6 x fp4 path, gives a wave two row tiles of weights: K ranges of 1, 3, 4, 5 and 9
    blocks (shorter than the copy ring, odd tails) and row-tile counts that leave a wave one or no live tile."""
    note(f"grouped two token tiles bits={bits} T={T}")
    common = dict(outlier_frac=0.01, outlier_scale=30.0)
    sites = [
        synth.Site("p_k128", T, 128, 32, hadamard=True, seed=61, **common),
        synth.Site("p_k384", T, 384, 96, hadamard=False, seed=62, **common),
        synth.Site("p_k512", T, 512, 160, hadamard=True, seed=63, **common),
        synth.Site("p_k640", T - 1, 640, 224, hadamard=False, seed=64, groups=1, **common),
        synth.Site("p_k1152", T, 1152, 288, hadamard=False, seed=65, groups=3, **common),
    ]
    run_group(hbl, sites, [bits] * len(sites))


def test_grouped_single_problem_and_fallbacks(hbl):
    """A group of one; a group with a large-T member, mixed bit widths or more than 8 problems runs
    problem by problem and must give the same results."""
    note("grouped single / fallbacks")
    common = dict(outlier_frac=0.01, outlier_scale=30.0)
    small = synth.Site("f_small", 5, 1024, 128, hadamard=True, seed=41, **common)
    big = synth.Site("f_big", 100, 1024, 128, hadamard=True, seed=42, **common)
    plain = synth.Site("f_plain", 7, 384, 64, hadamard=False, seed=43, **common)
    run_group(hbl, [small], [4])
    run_group(hbl, [small, big, plain], [4, 4, 4])
    run_group(hbl, [small, plain], [4, 8])
    run_group(hbl, [small, plain] * 5, [4] * 10)


def test_grouped_argument_errors(hbl):
    note("grouped errors")
    x = torch.zeros((4, 256), dtype=torch.bfloat16, device="cuda")
    packed = torch.zeros(hbl.packed_bytes(64, 256), dtype=torch.uint8, device="cuda")
    al = torch.ones(1, dtype=torch.float32, device="cuda")
    y = torch.empty((4, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(hbl.HblError) as e:
        hbl.bitlinear_forward_grouped([(x, packed, 64, al, 5, True, y)])
    assert e.value.status == hbl.E_BITS
    with pytest.raises(hbl.HblError) as e:
        hbl.bitlinear_forward_grouped([(x, packed, 64, al, 4, True, y)],
                                      workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == hbl.E_WORKSPACE
    with pytest.raises(hbl.HblError) as e:
        hbl.bitlinear_forward_grouped([(x[:, :192].contiguous(), packed, 64, al, 4, True, y)])
    assert e.value.status == hbl.E_SHAPE
    assert hbl.bitlinear_forward_grouped([]) == []


@pytest.mark.parametrize("K", [128, 256, 512, 1024, 2048, 4096, 8192, 16384])
@pytest.mark.parametrize("in_dtype", [synth.BF16, synth.F32])
def test_fwht_only_forward_and_backward(hbl, K, in_dtype):
    """The transform by itself (Eq. 3-4; Eq. 8 when applied to gradient rows): bit-exact against the
    oracle in fp32 and in bf16 output, and applying it twice returns the input."""
    note(f"fwht only K={K} in={in_dtype}")
    site = synth.Site("g", 37, K, 32, x_dtype=in_dtype, outlier_frac=0.01, outlier_scale=30.0, seed=900 + K)
    g = synth.make_x(site)
    gd = dev_x(g)
    want32 = O.hadamard_backward(g)
    got32 = hbl.fwht(gd)
    assert np.array_equal(got32.cpu().numpy().view(np.uint32), want32.view(np.uint32))
    got16 = hbl.fwht(gd, out_dtype=torch.bfloat16)
    assert np.array_equal(host_bf16_bits(got16), O.hadamard_backward(g, out_bf16=True))
    twice = hbl.fwht(got32).cpu().numpy()
    x32 = synth.bf16_bits_to_f32(g) if g.dtype == np.uint16 else g
    assert np.abs(twice - x32).max() <= 1e-5 * np.abs(x32).max() * math.log2(K)


def test_fwht_only_errors_and_empty(hbl):
    note("fwht only errors")
    x = torch.zeros((4, 384), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(hbl.HblError) as e:
        hbl.fwht(x)
    assert e.value.status == hbl.E_SHAPE
    assert hbl.fwht(torch.zeros((0, 256), dtype=torch.float32, device="cuda")).shape == (0, 256)


@pytest.mark.parametrize("K,T,dtype", [(16384, 700, synth.BF16), (4096, 4400, synth.BF16), (8192, 1500, synth.F32)])
def test_ln_quantiser_rows_walked_by_resident_workgroups(hbl, K, T, dtype):
    """The row-walking launch form with the RMS normalisation in front (its own instantiations of the kernel):
    several rows per workgroup, record form and byte form, all rows against the oracle."""
    note(f"row-walking ln quantiser K={K} T={T} {dtype}")
    g = ln_gain_for(K, K + T)
    site = synth.Site("a", T, K, 32, hadamard=True, x_dtype=dtype, outlier_frac=0.01, outlier_scale=30.0, seed=T)
    x = synth.make_x(site)
    c4, s4 = O.fwht_quant(O.rmsnorm(x, g, 1e-6), 4, hadamard=True, eps=EPS)
    xd, gd = dev_x(x), torch.from_numpy(g).cuda()
    rec, sd, cs = hbl.ln_fwht_quant(xd, gd, 1e-6, 4, True, EPS, code_offset=hbl.CODES_BF6)
    want = record_bits(encode_bf6_records(c4.astype(np.int32)), T, K)
    assert np.array_equal(record_bits(rec.cpu().numpy(), T, K), want)
    assert np.array_equal(sd.cpu().numpy(), s4) and np.array_equal(cs.cpu().numpy(), c4.astype(np.int32).sum(1))
    c, sd, cs = hbl.ln_fwht_quant(xd, gd, 1e-6, 4, True, EPS, code_offset=8)
    assert np.array_equal(c.cpu().numpy().astype(np.int32) - 8, c4.astype(np.int32))
    assert np.array_equal(sd.cpu().numpy(), s4) and np.array_equal(cs.cpu().numpy(), c4.astype(np.int32).sum(1))


def ln_gain_for(K, seed):
    """RMS-norm gains around 1 with a few large channels (the gains are where trained models park outliers)."""
    rng = np.random.default_rng(seed)
    g = (1.0 + 0.1 * rng.standard_normal(K)).astype(np.float32)
    g[rng.integers(0, K, 3)] *= 8.0
    return g


@pytest.mark.parametrize("K,hadamard", [(128, True), (512, True), (2048, True), (4096, True), (8192, True),
                                        (16384, True), (4096, False), (1536, False), (640, False)])
@pytest.mark.parametrize("bits", [4, 8])
def test_ln_fwht_quant_parity(hbl, K, hadamard, bits):
    """LN of Eq. 7 (RMS normalisation) fused ahead of the transform: codes and scales against the
    oracle's rmsnorm -> fwht_quant chain, every quantiser kernel family, both input types."""
    note(f"ln fwht_quant K={K} hadamard={hadamard} bits={bits}")
    g = ln_gain_for(K, K + bits)
    for dtype in (synth.BF16, synth.F32):
        site = synth.Site("a", 21, K, 32, hadamard=hadamard, x_dtype=dtype, outlier_frac=0.01, outlier_scale=30.0,
                          seed=K + 7 * bits)
        x = synth.make_x(site)
        xn = O.rmsnorm(x, g, 1e-6)
        c_ref, s_ref = O.fwht_quant(xn, bits, hadamard=hadamard, eps=EPS)
        codes, sd, cs = hbl.ln_fwht_quant(dev_x(x), torch.from_numpy(g).cuda(), 1e-6, bits, hadamard, EPS)
        check_codes(codes.cpu().numpy(), c_ref)
        assert np.array_equal(codes.cpu().numpy(), c_ref)
        assert np.array_equal(sd.cpu().numpy(), s_ref)
        assert np.array_equal(cs.cpu().numpy(), c_ref.astype(np.int32).sum(1))


@pytest.mark.parametrize("T,K,N,hadamard,bits", [(150, 4096, 288, True, 4), (150, 2048, 96, False, 4),
                                                 (40, 1024, 128, True, 8), (5, 4096, 544, False, 4),
                                                 (9, 16384, 64, True, 4)])
def test_ln_bitlinear_forward_and_grouped(hbl, T, K, N, hadamard, bits):
    """Whole call with the fused normalisation, on the prefill (fp6 x fp4 / int8) and small-batch
    paths, alone and as a member of a grouped call."""
    note(f"ln forward T={T} K={K} N={N} hadamard={hadamard} bits={bits}")
    site = synth.Site("a", T, K, N, hadamard=hadamard, outlier_frac=0.01, outlier_scale=30.0, seed=T + K)
    x = synth.make_x(site)
    g = ln_gain_for(K, T + K)
    wc_ref, al_ref, wc_d, al_d, packed = setup_weights(hbl, site)
    y_ref = O.bitlinear_forward(O.rmsnorm(x, g, 1e-6), wc_ref, al_ref, bits, hadamard, EPS)
    gd = torch.from_numpy(g).cuda()
    y = hbl.ln_bitlinear_forward(dev_x(x), gd, 1e-6, hadamard, packed, N, al_d, bits, EPS)
    assert np.array_equal(host_bf16_bits(y), y_ref)
    other = synth.Site("b", min(T, 64), 512, 64, hadamard=True, outlier_frac=0.01, outlier_scale=30.0, seed=77)
    xo = synth.make_x(other)
    wo_ref, ao_ref, _, ao_d, po = setup_weights(hbl, other)
    ys = hbl.bitlinear_forward_grouped([(dev_x(x), packed, N, al_d, bits, hadamard, None, gd, 1e-6),
                                        (dev_x(xo), po, other.N, ao_d, bits, True, None)], EPS)
    assert np.array_equal(host_bf16_bits(ys[0]), y_ref)
    assert np.array_equal(host_bf16_bits(ys[1]), O.bitlinear_forward(xo, wo_ref, ao_ref, bits, True, EPS))


@pytest.mark.parametrize("batch", [8, 40])
def test_grouped_call_in_a_hip_graph_replays_exactly(hbl, batch):
    """The grouped call captured into a HIP graph (kernel nodes only: its argument blocks travel as
    kernel arguments) and replayed with fresh inputs between replays, eager work and
    synchronisations in between: every replay must equal the eager result on the same inputs.
    At batch 40 the K = 16384 problem is split over workgroups, so every replay counts its arrivals in
    the same words of the library's counter array: they must be back at zero each time."""
    note(f"grouped call under graph replay, batch {batch}")
    common = dict(outlier_frac=0.01, outlier_scale=30.0)
    sites = [synth.Site("r_h", batch, 4096, 256, hadamard=True, seed=51, **common),
             synth.Site("r_p", batch, 1536, 160, hadamard=False, seed=52, groups=1, **common),
             synth.Site("r_big", batch, 16384, 192, hadamard=True, seed=53, **common)]
    packs = [setup_weights(hbl, s) for s in sites]
    xs = [dev_x(synth.make_x(s)) for s in sites]
    ys = [torch.empty((s.T, s.N), dtype=torch.bfloat16, device="cuda") for s in sites]
    items = [(xs[i], packs[i][4], s.N, packs[i][3], 4, s.hadamard, ys[i]) for i, s in enumerate(sites)]
    probs = hbl.make_problems(items)
    ws = torch.empty(hbl.grouped_workspace_bytes(probs, len(items)), dtype=torch.uint8, device="cuda")
    hbl.bitlinear_forward_grouped(items, EPS, workspace=ws, problems=probs)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            hbl.bitlinear_forward_grouped(items, EPS, workspace=ws, problems=probs)
    torch.cuda.synchronize()
    for rep in range(4):
        for i, s in enumerate(sites):      # new inputs in place (same buffers the graph captured)
            xs[i].copy_(dev_x(synth.make_x(synth.Site(s.name, s.T, s.K, s.N, hadamard=s.hadamard, seed=60 + rep, **common))))
        torch.cuda.synchronize()
        eager = [fn(xs[i], packs[i][4], s.N, packs[i][3], 4, EPS)
                 for i, s in enumerate(sites)
                 for fn in [hbl.hbitlinear_forward if s.hadamard else hbl.plain_bitlinear_forward]]
        torch.cuda.synchronize()
        for y in ys:
            y.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for y, e, s in zip(ys, eager, sites):
            assert torch.equal(y.view(torch.int16), e.view(torch.int16)), f"replay {rep}: {s.name}"


def test_weight_and_activation_rotation_variant(hbl):
    """The ablation's variant that rotates the weights too (offline): Q_w(W H) . Q(H x).  Built from
    the library's own pieces - hbl_fwht on the weight rows, then ternarise / pack, then the ordinary
    H-BitLinear forward - and equal, bit for bit, to the same chain in the oracle."""
    note("weight + activation rotation")
    site = synth.Site("rot", 70, 1024, 96, hadamard=True, outlier_frac=0.01, outlier_scale=30.0, seed=71)
    x, W = synth.make_x(site), synth.make_w(site)
    Wr_ref = O.fwht_rows(W)
    wc_ref, a_ref = O.ternarize_weights_absmean(Wr_ref, EPS)
    y_ref = O.hbitlinear_forward(x, wc_ref, np.array([a_ref], np.float32), 4, EPS)
    Wr = hbl.fwht(torch.from_numpy(W).cuda())
    assert np.array_equal(Wr.cpu().numpy().view(np.uint32), Wr_ref.view(np.uint32))
    wc, alpha = hbl.ternarize_weights_absmean(Wr, EPS)
    y = hbl.hbitlinear_forward(dev_x(x), hbl.pack_ternary_2bit(wc), site.N, alpha, 4, EPS)
    assert np.array_equal(host_bf16_bits(y), y_ref)


def _random_site(rng, i, t_max):
    hadamard = bool(rng.integers(0, 2))
    K = int(rng.choice([128, 256, 512, 1024, 2048, 4096, 8192])) if hadamard else 128 * int(rng.integers(1, 40))
    groups = int(rng.choice([1, 1, 2, 3]))
    N = 32 * groups * int(rng.integers(1, 7))
    T = int(rng.integers(1, t_max + 1))
    dtype = synth.BF16 if rng.integers(0, 4) else synth.F32
    return synth.Site(f"rnd{i}", T, K, N, hadamard=hadamard, groups=groups, x_dtype=dtype, outlier_frac=0.01,
                      outlier_scale=float(rng.choice([1.0, 30.0])), seed=1000 + i)


@pytest.mark.parametrize("seed", range(6))
def test_random_shapes_single_and_grouped(hbl, seed):
    """Seeded random shapes (token counts on both sides of every path switch, ragged feature counts,
    scale groups, both input types and bit widths): every single call and one grouped call per
    draw, bit for bit against the oracle."""
    rng = np.random.default_rng(4242 + seed)
    bits = int(rng.choice([4, 8]))
    sites = [_random_site(rng, 10 * seed + i, t_max=[4, 16, 40, 64, 130, 300][seed]) for i in range(5)]
    note(f"random shapes seed={seed} bits={bits}: " + ", ".join(f"{s.T}x{s.K}->{s.N}{'H' if s.hadamard else 'P'}" for s in sites))
    # a grouped call needs one input type: group the bf16 sites, run the others alone
    main = [s for s in sites if s.x_dtype == synth.BF16]
    run_group(hbl, main, [bits] * len(main))
    for s in sites:
        if s.x_dtype != synth.BF16:
            run_group(hbl, [s], [bits])


def test_offsets_beyond_two_to_the_31(hbl):
    """T * K = 2.3e9 elements: any 32-bit element offset in a kernel would wrap.  Inputs are drawn on the
    GPU (4.6 GB of bf16); the oracle checks sampled rows around the wrap points and at both ends."""
    note("offsets beyond 2^31")
    T, K, N = 140000, 16384, 64
    g = torch.Generator(device="cuda")
    g.manual_seed(3)
    x = torch.randn((T, K), device="cuda", generator=g).to(torch.bfloat16)
    W = (np.random.default_rng(5).standard_normal((N, K)) * 0.02).astype(np.float32)
    wc_ref, a_ref = O.ternarize_weights_absmean(W, EPS)
    wc, alpha = hbl.ternarize_weights_absmean(torch.from_numpy(W).cuda(), EPS)
    packed = hbl.pack_ternary_2bit(wc)
    rows = np.r_[0:40, 65530:65560, 131060:131090, T - 40:T]
    rows_d = torch.from_numpy(rows).cuda()
    xs = x[rows_d].view(torch.int16).cpu().numpy().view(np.uint16)
    for bits, hadamard in ((4, True), (8, False)):
        fn = hbl.hbitlinear_forward if hadamard else hbl.plain_bitlinear_forward
        y = fn(x, packed, N, alpha, bits, EPS)
        ref = O.bitlinear_forward(xs, wc_ref, np.array([a_ref], np.float32), bits, hadamard, EPS)
        assert np.array_equal(host_bf16_bits(y[rows_d]), ref), (bits, hadamard)
        del y
    del x
    torch.cuda.empty_cache()


# --- low-bit Q/K/V head states (Section 3.1) -----------------------------------------------------------

@pytest.mark.parametrize("bits", [8, 4, 3])
@pytest.mark.parametrize("d,rows,dtype", [(128, 4100, synth.BF16), (64, 333, synth.BF16), (256, 77, synth.F32),
                                          (32, 1030, synth.F32), (512, 65, synth.BF16)])
def test_kv_quant_absmax_parity(hbl, bits, d, rows, dtype):
    """Per-head absmax quantiser of the attention states: the packed stream and the scales bit for bit against
    the oracle, then the inverse map in both output types; row counts that leave a ragged last workgroup."""
    note(f"kv quant bits={bits} d={d} rows={rows} {dtype}")
    rng = np.random.default_rng(1000 * bits + d + rows)
    x = rng.standard_normal((rows, d)).astype(np.float32) * np.exp(rng.standard_normal((rows, 1))).astype(np.float32)
    x[:, d // 3] *= 15.0                      # an outlier channel, as key states have
    x[rows // 2] = 0.0                        # an all-zero head
    xh = synth.f32_to_bf16_bits(x) if dtype == synth.BF16 else x
    codes, packed_ref, s_ref = O.kv_quant_absmax(xh, bits, EPS)
    packed, scales = hbl.kv_quant_absmax(dev_x(xh), bits, EPS)
    assert packed.shape == (rows, d * bits // 8)
    assert np.array_equal(packed.cpu().numpy(), packed_ref)
    assert np.array_equal(scales.cpu().numpy(), s_ref)
    out32 = hbl.kv_dequant(packed, scales, d, bits, out_dtype=torch.float32)
    assert np.array_equal(out32.cpu().numpy(), O.kv_dequant(codes, s_ref, bits))
    out16 = hbl.kv_dequant(packed, scales, d, bits, out_dtype=torch.bfloat16)
    assert np.array_equal(host_bf16_bits(out16), O.kv_dequant(codes, s_ref, bits, out_bf16=True))


def test_kv_quant_errors_and_empty(hbl):
    note("kv quant errors")
    x = torch.zeros((4, 96), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(hbl.HblError):
        hbl.kv_quant_absmax(x, 4)                                   # head size not supported
    x = torch.zeros((4, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(hbl.HblError):
        hbl.kv_quant_absmax(x, 5)
    p, s = hbl.kv_quant_absmax(x[:0], 4)
    assert p.shape[0] == 0 and s.shape[0] == 0
    p, s = hbl.kv_quant_absmax(x, 3)                                # zero rows of data: every code is the offset
    torch.cuda.synchronize()
    assert np.array_equal(np.unpackbits(p.cpu().numpy(), axis=1, bitorder="little").reshape(4, 128, 3),
                          np.broadcast_to(np.array([0, 0, 1], np.uint8), (4, 128, 3)))
    assert np.all(s.cpu().numpy() == 0.0)


def test_binding_rejects_short_buffers_before_the_library_sees_them(hbl):
    """The binding checks what the library cannot see through raw pointers: a packed-weight buffer or an output
    too small for the stated N would be read or written out of bounds on the device."""
    note("binding validation")
    x = torch.zeros((4, 256), dtype=torch.bfloat16, device="cuda")
    al = torch.ones(1, dtype=torch.float32, device="cuda")
    good = torch.zeros(hbl.packed_bytes(64, 256), dtype=torch.uint8, device="cuda")
    with pytest.raises(ValueError):
        hbl.hbitlinear_forward(x, good[:-16], 64, al, 4)
    with pytest.raises(ValueError):
        hbl.hbitlinear_forward(x, good, 128, al, 4)                               # packed for 64 rows, N says 128
    with pytest.raises(ValueError):
        hbl.hbitlinear_forward(x, good, 64, al, 4, y=torch.empty((4, 32), dtype=torch.bfloat16, device="cuda"))
    with pytest.raises(ValueError):
        hbl.hbitlinear_forward(x, good, 64, al.double(), 4)
    with pytest.raises(ValueError):
        hbl.bitlinear_forward_grouped([(x, good, 128, al, 4, True, None)])
    assert hbl.hbitlinear_forward(x, good, 64, al, 4).shape == (4, 64)
