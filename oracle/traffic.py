"""Memory-transfer model of Sec. 6: bits moved per convolution layer.

eq. (4): static quantization moves the weights, the input feature map and the
low-bit output once.  eq. (5): dynamic quantization moves the weights and input,
saves the accumulator output at b_acc bits, loads it again, and saves the
low-bit output.  For depthwise layers the weight term is C * k^2 (one filter per
channel): with C_in * C_out * k^2 the depthwise rows of Table 5 do not come out.

Test infrastructure, like the rest of this package.  Pinned by the values
printed in Table 5.
"""


def weight_elems(c_in, c_out, k, depthwise=False):
    return c_in * k * k if depthwise else c_in * c_out * k * k


def static_bits(c_in, c_out, k, w, h, b_w=8, b_a=8, depthwise=False, batch=1):
    """eq. (4)."""
    return (weight_elems(c_in, c_out, k, depthwise) * b_w
            + batch * c_in * w * h * b_a
            + batch * c_out * w * h * b_a)


def dynamic_bits(c_in, c_out, k, w, h, b_w=8, b_a=8, b_acc=32, depthwise=False, batch=1):
    """eq. (5)."""
    return (weight_elems(c_in, c_out, k, depthwise) * b_w
            + batch * c_in * w * h * b_a
            + batch * c_out * w * h * b_acc      # save accumulator output
            + batch * c_out * w * h * b_acc      # load accumulator output
            + batch * c_out * w * h * b_a)       # save quantized output


def kib(bits):
    """Table 5 prints KB = 1024 bytes."""
    return bits / 8.0 / 1024.0
