"""Host-side logic of the stack driver (no GPU)."""
from paper_2602_07899_amd import stack as gstack


def test_second_moment_choice_follows_the_flop_model():
    pays = gstack.second_moment_pays
    # 13B-class layer on 153,600 tokens: every group
    assert pays(153600, 5120, [5120, 5120, 5120], 20) and pays(153600, 5120, [5120], 20)
    assert pays(153600, 5120, [13824, 13824], 20) and pays(153600, 13824, [5120], 20)
    # 7B-class layer on 10,240 tokens: the attention and gate/up groups, not the 11008-deep down_proj
    assert pays(10240, 4096, [4096] * 3, 20) and pays(10240, 4096, [11008, 11008], 20)
    assert not pays(10240, 11008, [4096], 20)
    # fewer tokens than channels never pays; with one candidate the matrix alone costs half of the
    # token form on a square layer, so it takes at least two
    assert not pays(256, 512, [512], 20)
    assert not pays(40960, 4096, [4096], 1) and pays(40960, 4096, [4096], 2)
