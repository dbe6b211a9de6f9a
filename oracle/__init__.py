"""CPU oracle for fused fake quantization.  Test infrastructure only: the product
package never imports this."""
