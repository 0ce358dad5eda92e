"""CPU oracle of the MoE expert layer -- test infrastructure only.

Only tests, the smoke check and the bench's CPU-baseline leg may import this
package; the product (paper_2402_07033_amd) never does.
"""
