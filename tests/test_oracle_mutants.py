"""The pins must be able to tell a wrong oracle from the right one: each case
plants one plausible mistake in a copy of the oracle's C source (on the CPU, in a
temporary build), points the pin tests at that build and expects at least one of
them to fail.  The unmodified source, built the same way, must pass them all."""
import os
import subprocess
import tempfile

import pytest

from oracle import build as obuild
from oracle import oracle as orc
from tests import test_oracle_pins as pins

MUTANTS = {
    "lstm gates f and g swapped":
        ("double gf = sigmoid(g[hid + u]);\n        double gg = tanh(g[2 * hid + u]);",
         "double gf = sigmoid(g[2 * hid + u]);\n        double gg = tanh(g[hid + u]);"),
    "lstm recurrent term dropped":
        ("for (int k = 0; k < hid; ++k) s += (double)W_hh[(size_t)r * hid + k] * h[k];", ""),
    "lstm bias dropped":
        ("double s = (double)b[r];", "double s = 0.0;"),
    "lstm h uses old cell":
        ("c[u] = gf * c[u] + gi * gg;\n        h[u] = go * tanh(c[u]);",
         "h[u] = go * tanh(c[u]);\n        c[u] = gf * c[u] + gi * gg;"),
    "convolution flipped":
        ("int jj = j + k - pad;", "int jj = j - k + pad;"),
    "convolution padding off by one":
        ("int pad = (ksz - 1) / 2;", "int pad = (ksz - 1) / 2 + 1;"),
    "location channels swapped":
        ("memcpy(u, w_last, sizeof(double) * L);\n        memcpy(u + L, w_acc, sizeof(double) * L);",
         "memcpy(u, w_acc, sizeof(double) * L);\n        memcpy(u + L, w_last, sizeof(double) * L);"),
    "energy without query":
        ("tanh(q[a] + pl + PM[(size_t)j * A + a])", "tanh(pl + PM[(size_t)j * A + a])"),
    "energy without location term":
        ("tanh(q[a] + pl + PM[(size_t)j * A + a])", "tanh(q[a] + PM[(size_t)j * A + a])"),
    "softmax not normalised":
        ("for (int j = 0; j < L; ++j) w[j] /= den;", ""),
    "memory projection transposed":
        ("s += (double)mem_w[a * d->enc_dim + k] * (double)F[(size_t)j * d->enc_dim + k];",
         "s += (double)mem_w[(k * d->att_dim + a) % (d->att_dim * d->enc_dim)] * (double)F[(size_t)j * d->enc_dim + k];"),
    "context uses transposed weights index":
        ("for (int j = 0; j < L; ++j) s += w[j] * (double)F[(size_t)j * d->enc_dim + k];",
         "for (int j = 0; j < L; ++j) s += w[L - 1 - j] * (double)F[(size_t)j * d->enc_dim + k];"),
    "prenet second relu missing":
        ("p[o] = s > 0.0 ? s : 0.0;", "p[o] = s;"),
    "prenet first layer transposed":
        ("s += (double)W1[o * d->n_mel + i] * m[i];", "s += (double)W1[(i * d->prenet_dim + o) % (d->prenet_dim * d->n_mel)] * m[i];"),
    "projection concatenation swapped":
        ("for (int k = 0; k < H; ++k) s += (double)W->mel_w[(size_t)o * IN + k] * h_dec[k];\n"
         "        for (int k = 0; k < E; ++k) s += (double)W->mel_w[(size_t)o * IN + H + k] * ctx[k];",
         "for (int k = 0; k < E; ++k) s += (double)W->mel_w[(size_t)o * IN + k] * ctx[k];\n"
         "        for (int k = 0; k < H; ++k) s += (double)W->mel_w[(size_t)o * IN + E + k] * h_dec[k];"),
    "attention lstm input order swapped":
        ("orc_prenet(d, r->W.prenet1, r->W.prenet2, r->m, x);\n    memcpy(x + d->prenet_dim, r->a, sizeof(double) * d->enc_dim);",
         "orc_prenet(d, r->W.prenet1, r->W.prenet2, r->m, x + d->enc_dim);\n    memcpy(x, r->a, sizeof(double) * d->enc_dim);"),
    "decoder lstm sees previous context":
        ("memcpy(x, r->h_att, sizeof(double) * d->att_rnn_dim);\n    memcpy(x + d->att_rnn_dim, r->a, sizeof(double) * d->enc_dim);\n    orc_lstm_cell(dec_in",
         "orc_lstm_cell(dec_in"),
    "accumulated weights updated before attention":
        ("    /* A, W_last = LSA(H_att, F_enc, W_acc) */\n", "    for (int j = 0; j < r->L; ++j) r->w_acc[j] += r->w_last[j];\n"),
    "accumulated weights not updated":
        ("r->w_acc[j] += w[j];", ""),
    "last weights not carried":
        ("r->w_last[j] = w[j];", ""),
    "mel not fed back":
        ("orc_projection(d, &r->W, r->h_dec, r->a, r->m, &stop);",
         "{ double tmp[512]; orc_projection(d, &r->W, r->h_dec, r->a, tmp, &stop); if (mel_out) memcpy(mel_out, tmp, sizeof(double) * d->n_mel); mel_out = NULL; }"),
    "stop rule inverted":
        ("sigmoid(stop) > r->stop_threshold", "sigmoid(stop) < r->stop_threshold"),
    "bf16 rounding truncates":
        ("u = (u + 0x7FFFu + lsb) & 0xFFFF0000u;", "u = u & 0xFFFF0000u;"),
}

# every pin except the two slow full-size ones
PIN_TESTS = [
    lambda: pins.test_lstm_zero_weights_closed_form(),
    lambda: pins.test_lstm_matches_library_cell(1),
    lambda: [pins.test_location_delta_kernel_shifts(s, c) for s in (-15, -3, 0, 4, 15) for c in (0, 1)],
    lambda: [pins.test_location_matches_library_conv(L, n) for L in (1, 5, 31, 32, 67) for n in (1, 2)],
    lambda: pins.test_location_brute_force_tiny(),
    lambda: pins.test_lsa_softmax_invariants_and_convexity(),
    lambda: pins.test_lsa_v_zero_gives_uniform_weights_and_column_mean(),
    lambda: pins.test_lsa_without_query_and_location_is_softmax_of_v_tanh_pm(),
    lambda: pins.test_lsa_energy_formula_against_numpy_and_library(),
    lambda: pins.test_lsa_channel_order_last_then_acc(),
    lambda: pins.test_memory_projection_and_bf16_rounding(),
    lambda: pins.test_prenet_identity_like_weights_relu(),
    lambda: pins.test_projection_one_hot_rows_pick_h_then_ctx(),
    lambda: [pins.test_request_matches_library_composition(n) for n in (1, 2)],
    lambda: pins.test_concatenation_orders_with_one_hot_probes(),
    lambda: pins.test_step_order_acc_updated_after_attention(),
    lambda: pins.test_snapshot_resume(),
    lambda: pins.test_stop_threshold_ends_request_and_keeps_tripping_frame(),
    lambda: pins.test_pool_decode_is_each_request_alone_and_thread_invariant(),
]


def _build_variant(src_text: str, workdir: str, name: str):
    c = os.path.join(workdir, name + ".c")
    so = os.path.join(workdir, name + ".so")
    with open(c, "w") as f:
        f.write(src_text)
    subprocess.run(["gcc", "-O1", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-w", "-o", so, c, obuild.SRC_POSTNET,
                    obuild.SRC_VOCODER, obuild.SRC_ENCODER, "-lm"], check=True)
    return orc.load(so)


def _pins_fail(lib, tests=None) -> bool:
    prev = orc.use_library(lib)
    try:
        for t in (PIN_TESTS if tests is None else tests):
            try:
                t()
            except (AssertionError, ValueError):
                return True
        return False
    finally:
        orc.use_library(prev)


@pytest.fixture(scope="module")
def source():
    return open(obuild.SRC).read()


def test_unmodified_source_passes_every_pin(source):
    with tempfile.TemporaryDirectory() as tmp:
        assert not _pins_fail(_build_variant(source, tmp, "clean"))


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_planted_mistake(name, source):
    old, new = MUTANTS[name]
    assert source.count(old) == 1, f"mutation site for '{name}' not found exactly once"
    with tempfile.TemporaryDirectory() as tmp:
        lib = _build_variant(source.replace(old, new), tmp, "mutant")
        assert _pins_fail(lib), f"no pin noticed: {name}"


# ---- the vocoder oracle (oracle/vocoder_oracle.c), same method
from tests import test_vocoder_oracle as vpins

VOCODER_MUTANTS = {
    "convolution flipped":
        ("int tt = t + (j - half) * dil;", "int tt = t - (j - half) * dil;"),
    "dilation ignored":
        ("int tt = t + (j - half) * dil;", "int tt = t + (j - half);"),
    "convolution bias dropped":
        ("double s = (double)b[co];\n            for (int ci = 0; ci < c_in; ++ci)\n                for (int j = 0; j < k; ++j) {\n                    int tt = t + (j - half) * dil;",
         "double s = 0.0;\n            for (int ci = 0; ci < c_in; ++ci)\n                for (int j = 0; j < k; ++j) {\n                    int tt = t + (j - half) * dil;"),
    "transposed convolution padding dropped":
        ("int o = t * stride + j - pad;", "int o = t * stride + j;"),
    "transposed convolution weight transposed":
        ("w[((size_t)ci * c_out + co) * k + j] * xv", "w[(((size_t)co * c_in + ci) * k + j) % ((size_t)c_in * c_out * k)] * xv"),
    "residual connection dropped":
        ("for (size_t q = 0; q < n; ++q) x[q] += t[q];", "for (size_t q = 0; q < n; ++q) x[q] = t[q];"),
    "second convolution of a pair dilated too":
        ("orc_conv1d(T, c, c, k, 1, w[2 * i + 1], b[2 * i + 1], a, t);", "orc_conv1d(T, c, c, k, dils[i], w[2 * i + 1], b[2 * i + 1], a, t);"),
    "no activation before the second convolution":
        ("orc_leaky_relu(n, slope, t, a);\n        orc_conv1d(T, c, c, k, 1,", "memcpy(a, t, sizeof(double) * n);\n        orc_conv1d(T, c, c, k, 1,"),
    "blocks summed, not averaged":
        ("for (size_t q = 0; q < n_out; ++q) acc[q] /= (double)g->n_blocks;", ""),
    "blocks chained instead of parallel":
        ("memcpy(r, y, sizeof(double) * n_out);\n            orc_resblock(", "if (bk == 0) memcpy(r, y, sizeof(double) * n_out);\n            orc_resblock("),
    "no activation before the upsampling":
        ("orc_leaky_relu(n_in, g->slope, x, a);\n        orc_conv_transpose1d(", "memcpy(a, x, sizeof(double) * n_in);\n        orc_conv_transpose1d("),
    "no tanh at the output":
        ("audio[t] = tanh(audio[t]);", "audio[t] = audio[t];"),
    "leaky slope applied to positives":
        ("y[i] = x[i] > 0.0 ? x[i] : slope * x[i];", "y[i] = x[i] < 0.0 ? x[i] : slope * x[i];"),
    "fade sampled at the left edge":
        ("double u = ((double)i + 0.5) / (double)n;", "double u = ((double)i) / (double)n;"),
    "fade coefficients swapped":
        ("fused[i] = al[i] * head_cur[i] + be[i] * tail_pre[i];", "fused[i] = be[i] * head_cur[i] + al[i] * tail_pre[i];"),
    "linear fade":
        ("alpha[i] = sin(0.5 * ORC_PI * u);\n        beta[i] = cos(0.5 * ORC_PI * u);", "alpha[i] = u;\n        beta[i] = 1.0 - u;"),
}

VOCODER_PINS = [
    lambda: [vpins.test_conv1d_equals_library_routine(*a) for a in ((3, 5, 3, 1, 11), (8, 8, 7, 3, 40), (4, 2, 11, 5, 23))],
    lambda: [vpins.test_conv_transpose1d_equals_library_routine(*a) for a in ((4, 2, 8, 7), (6, 3, 2, 13))],
    lambda: vpins.test_conv1d_impulse_by_hand(),
    lambda: vpins.test_conv_transpose1d_impulse_by_hand(),
    lambda: vpins.test_generator_equals_composition_of_library_routines(),
    lambda: vpins.test_fade_is_equal_power(),
    lambda: vpins.test_crossfade_by_hand(),
    lambda: vpins.test_stream_tiles_the_utterance_and_follows_eq3_eq4(),
]


def _build_vocoder_variant(src_text: str, workdir: str, name: str):
    c = os.path.join(workdir, name + ".c")
    so = os.path.join(workdir, name + ".so")
    with open(c, "w") as f:
        f.write(src_text)
    subprocess.run(["gcc", "-O1", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-w", "-o", so, obuild.SRC, obuild.SRC_POSTNET,
                    c, obuild.SRC_ENCODER, "-lm"], check=True)
    return orc.load(so)


@pytest.fixture(scope="module")
def vocoder_source():
    return open(obuild.SRC_VOCODER).read()


def test_unmodified_vocoder_source_passes_every_pin(vocoder_source):
    with tempfile.TemporaryDirectory() as tmp:
        assert not _pins_fail(_build_vocoder_variant(vocoder_source, tmp, "clean"), VOCODER_PINS)


@pytest.mark.parametrize("name", sorted(VOCODER_MUTANTS))
def test_vocoder_pins_catch_planted_mistake(name, vocoder_source):
    old, new = VOCODER_MUTANTS[name]
    assert vocoder_source.count(old) == 1, f"mutation site for '{name}' not found exactly once"
    with tempfile.TemporaryDirectory() as tmp:
        lib = _build_vocoder_variant(vocoder_source.replace(old, new), tmp, "mutant")
        assert _pins_fail(lib, VOCODER_PINS), f"no pin noticed: {name}"


# ---- the encoder oracle (oracle/encoder_oracle.c), same method
from tests import test_encoder_oracle as epins

ENCODER_MUTANTS = {
    "one embedding table left out":
        ("for (int t = 0; t < n_tables; ++t) s +=", "for (int t = 0; t < n_tables - 1; ++t) s +="),
    "every id sequence reads the token table":
        ("tables[t][(size_t)ids[t][j] * dim + d]", "tables[0][(size_t)(ids[t][j] % 3) * dim + d]"),
    "convolution flipped":
        ("int jj = j + k - half;", "int jj = j - k + half;"),
    "no relu":
        ("y[(size_t)j * c_out + co] = s > 0.0 ? s : 0.0;", "y[(size_t)j * c_out + co] = s;"),
    "convolution bias dropped":
        ("double s = (double)b[co];", "double s = 0.0;"),
    "backward direction runs forwards":
        ("for (int j = L - 1; j >= 0; --j) {", "for (int j = 0; j < L; ++j) {"),
    "backward direction keeps the forward state":
        ("    memset(h, 0, sizeof(double) * hid);\n    memset(c, 0, sizeof(double) * hid);\n", ""),
    "halves of the output swapped":
        ("memcpy(out + (size_t)j * 2 * hid, h, sizeof(double) * hid);\n    }\n    memset",
         "memcpy(out + (size_t)j * 2 * hid + hid, h, sizeof(double) * hid);\n    }\n    memset"),
    "backward direction uses the forward weights":
        ("orc_lstm_cell(in_dim, hid, W_ih_b, W_hh_b, b_b,", "orc_lstm_cell(in_dim, hid, W_ih_f, W_hh_f, b_f,"),
    "one convolution layer skipped":
        ("for (int l = 0; l < n_conv; ++l) {", "for (int l = 1; l < n_conv; ++l) {"),
}

ENCODER_PINS = [
    lambda: epins.test_embedding_sum_is_indexing(),
    lambda: [epins.test_conv_relu_equals_library_routine(L) for L in (1, 5, 23)],
    lambda: epins.test_conv_orientation_by_hand(),
    lambda: [epins.test_bilstm_equals_library_routine(L) for L in (1, 9)],
    lambda: epins.test_bilstm_directions_mirror_each_other(),
    lambda: epins.test_bilstm_zero_weights_closed_form(),
    lambda: [epins.test_encoder_equals_composition_of_library_routines(L) for L in (1, 30)],
]


def _build_encoder_variant(src_text: str, workdir: str, name: str):
    c = os.path.join(workdir, name + ".c")
    so = os.path.join(workdir, name + ".so")
    with open(c, "w") as f:
        f.write(src_text)
    subprocess.run(["gcc", "-O1", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-w", "-o", so, obuild.SRC, obuild.SRC_POSTNET,
                    obuild.SRC_VOCODER, c, "-lm"], check=True)
    return orc.load(so)


@pytest.fixture(scope="module")
def encoder_source():
    return open(obuild.SRC_ENCODER).read()


def test_unmodified_encoder_source_passes_every_pin(encoder_source):
    with tempfile.TemporaryDirectory() as tmp:
        assert not _pins_fail(_build_encoder_variant(encoder_source, tmp, "clean"), ENCODER_PINS)


@pytest.mark.parametrize("name", sorted(ENCODER_MUTANTS))
def test_encoder_pins_catch_planted_mistake(name, encoder_source):
    old, new = ENCODER_MUTANTS[name]
    assert encoder_source.count(old) == 1, f"mutation site for '{name}' not found exactly once"
    with tempfile.TemporaryDirectory() as tmp:
        lib = _build_encoder_variant(encoder_source.replace(old, new), tmp, "mutant")
        assert _pins_fail(lib, ENCODER_PINS), f"no pin noticed: {name}"


# ---- the PostNet oracle (oracle/postnet_oracle.c), same method
from tests import test_postnet_oracle as ppins

POSTNET_MUTANTS = {
    "convolution flipped":
        ("int tt = t + k - ORC_PN_TAPS / 2;", "int tt = t - k + ORC_PN_TAPS / 2;"),
    "padding off by one":
        ("int tt = t + k - ORC_PN_TAPS / 2;", "int tt = t + k - ORC_PN_TAPS / 2 - 1;"),
    "bias dropped":
        ("double s = (double)b[co];", "double s = 0.0;"),
    "weights transposed":
        ("w[((size_t)co * c_in + ci) * ORC_PN_TAPS + k]", "w[(((size_t)ci * c_out + co) * ORC_PN_TAPS + k) % ((size_t)c_in * c_out * ORC_PN_TAPS)]"),
    "tanh after the last layer too":
        ("orc_conv5(T, c_in, c_out, w[l], b[l], cur, l != n_layers - 1, nxt);", "orc_conv5(T, c_in, c_out, w[l], b[l], cur, 1, nxt);"),
    "no tanh between layers":
        ("orc_conv5(T, c_in, c_out, w[l], b[l], cur, l != n_layers - 1, nxt);", "orc_conv5(T, c_in, c_out, w[l], b[l], cur, 0, nxt);"),
    "residual sum dropped":
        ("out[i] = mel[i] + cur[i];", "out[i] = cur[i];"),
    "one layer skipped":
        ("for (int l = 0; l < n_layers; ++l) {\n        int c_in = l == 0 ? n_mel : channels;",
         "for (int l = 0; l < n_layers; ++l) {\n        if (l == 1) continue;\n        int c_in = l == 0 ? n_mel : channels;"),
    "chunk taken from the wrong end":
        ("memcpy(out, all + (size_t)s * n_mel,", "memcpy(out, all,"),
}

POSTNET_PINS = [
    lambda: [ppins.test_stack_equals_library_convolutions(T) for T in (1, 5, 23)],
    lambda: ppins.test_single_layer_delta_kernels_shift_with_zero_fill(),
    lambda: ppins.test_bias_and_channel_order(),
    lambda: ppins.test_centre_tap_identity_stack_closed_form(),
    lambda: ppins.test_last_chunk_equals_whole_utterance_and_chunks_tile(),
    lambda: ppins.test_receptive_field_of_a_chunk(),
]


def _build_postnet_variant(src_text: str, workdir: str, name: str):
    c = os.path.join(workdir, name + ".c")
    so = os.path.join(workdir, name + ".so")
    with open(c, "w") as f:
        f.write(src_text)
    subprocess.run(["gcc", "-O1", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-w", "-o", so, obuild.SRC, c,
                    obuild.SRC_VOCODER, obuild.SRC_ENCODER, "-lm"], check=True)
    return orc.load(so)


@pytest.fixture(scope="module")
def postnet_source():
    return open(obuild.SRC_POSTNET).read()


def test_unmodified_postnet_source_passes_every_pin(postnet_source):
    with tempfile.TemporaryDirectory() as tmp:
        assert not _pins_fail(_build_postnet_variant(postnet_source, tmp, "clean"), POSTNET_PINS)


@pytest.mark.parametrize("name", sorted(POSTNET_MUTANTS))
def test_postnet_pins_catch_planted_mistake(name, postnet_source):
    old, new = POSTNET_MUTANTS[name]
    assert postnet_source.count(old) == 1, f"mutation site for '{name}' not found exactly once"
    with tempfile.TemporaryDirectory() as tmp:
        lib = _build_postnet_variant(postnet_source.replace(old, new), tmp, "mutant")
        assert _pins_fail(lib, POSTNET_PINS), f"no pin noticed: {name}"
