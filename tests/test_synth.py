"""The seeded input generators and manifests (no arithmetic of the method): shapes, counts and id recipes."""
import numpy as np

import dp_synth as syn


def test_parameter_counts_of_the_workload_manifests():
    assert syn.manifest_param_count(syn.CONFIGS["C2"]["manifest"]()) == 85_054_464
    assert syn.manifest_param_count(syn.CONFIGS["C3"]["manifest"]()) == 334_088_192
    # with the token-type table (2 x 1024) and the embedding LayerNorm (2 x 1024)
    assert syn.manifest_param_count(syn.bert_manifest(24, 1024, 4096, 30522, 512, type_vocab=2)) == 334_092_288


def test_id_recipes():
    assert syn.segment_ids(2, 7).tolist() == [[0, 0, 0, 0, 1, 1, 1]] * 2
    assert syn.position_ids(2, 3).tolist() == [[0, 1, 2]] * 2
    ids = syn.zipf_ids(64, 128, 30522, 1.1, 5)
    assert ids.dtype == np.int32 and ids.min() >= 0 and ids.max() < 30522
    top = np.bincount(ids.reshape(-1)).max() / ids.size
    assert 0.10 < top < 0.18          # the most frequent id holds about 14 % of the tokens


def test_embedding_stage_shares_one_output_gradient():
    man = syn.bert_manifest(1, 16, 32, vocab=11, max_pos=8, type_vocab=2)
    layers = syn.device_layer_inputs(man, 3, 8, dtype="f32", act_std=1.0, grad_std=0.1, data_seed=3, device="cpu")
    assert [l["name"] for l in layers[:4]] == ["emb.tok", "emb.pos", "emb.type", "emb.ln"]
    assert layers[0]["G"] is layers[1]["G"] and layers[1]["G"] is layers[2]["G"]
    assert layers[3]["G"] is not layers[0]["G"]
    assert layers[2]["ids"].tolist()[0] == [0, 0, 0, 0, 1, 1, 1, 1] and layers[2]["V"] == 2
